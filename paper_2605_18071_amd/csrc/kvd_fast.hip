// Stages 1b, 2a and 2b of the decode step in one launch, one block of 1024 threads per unit:
// Top-K selection of the scored pages, the cache-directory update and the fetch of the unit's
// missed pages from the pinned host store (see kvd_selres_body.h).
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_selres_body.h"

namespace kvd {

constexpr int kFastThreads = 1024;

template <int IPT, bool DO_SELECT, bool DO_RESOLVE>
__global__ __launch_bounds__(kFastThreads) void select_resolve_kernel(FastArgs a) {
  __shared__ FastSmem<kFastThreads> sm;
  select_resolve_body<kFastThreads, IPT, DO_SELECT, DO_RESOLVE, false>(a, blockIdx.x + a.u0, sm);
}

template <bool SEL, bool RES>
static void launch_fast(int ipt, const FastArgs& a, int n_units, hipStream_t s) {
  dim3 grid(n_units), block(kFastThreads);
  if (ipt <= 4)
    hipLaunchKernelGGL((select_resolve_kernel<4, SEL, RES>), grid, block, 0, s, a);
  else if (ipt <= 8)
    hipLaunchKernelGGL((select_resolve_kernel<8, SEL, RES>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((select_resolve_kernel<16, SEL, RES>), grid, block, 0, s, a);
}

}  // namespace kvd

bool kvd_fast_path_ok(const kvd_ctx* c) {
  return !c->generic_select && c->NP <= KVD_FAST_MAX_PAGES && c->Cmax <= KVD_FAST_MAX_CAPACITY;
}

kvd::FastArgs kvd_fast_args(kvd_ctx* c, int layer, int step, bool do_gather, const float* scores, int32_t* sel_pages,
                            int32_t* sel_slots, int32_t* hit_mask, int32_t* evicted, int32_t* counts, int u0) {
  kvd::FastArgs a;
  const size_t lu = (size_t)layer * c->U;
  a.scores = scores;
  a.seq_len = c->d_seq_len;
  a.sel_pages = sel_pages;
  a.capacity = c->d_capacity + lu;
  a.resident = c->d_resident + lu;
  a.slot_page = c->d_slot_page + lu * c->Cmax;
  a.slot_stamp = c->d_slot_stamp + lu * c->Cmax;
  a.sel_slots = sel_slots;
  a.sel_entry = c->d_sel_entry;
  a.hit_mask = hit_mask;
  a.evicted = evicted;
  a.counts = counts;
  a.miss_list = c->d_miss_list;
  a.miss_count = c->d_miss_count;
  a.stats = c->d_stats;
  a.store = c->store_dev ? c->store_dev + (size_t)(layer % c->Lp) * c->U * c->NP * c->page_bytes : nullptr;
  a.pool = c->pool ? c->pool + lu * c->Cmax * c->page_bytes : nullptr;
  a.NP = c->NP; a.P = c->P; a.k = c->k; a.Cmax = c->Cmax;
  a.sink = c->cfg.sink_pages; a.recent = c->cfg.recent_pages; a.Hkv = c->Hkv; a.step = step; a.u0 = u0;
  a.do_gather = (do_gather && a.store && a.pool) ? 1 : 0;
  a.tiled = c->tiled;
  a.lookahead = c->cfg.policy == KVD_EVICT_LOOKAHEAD ? 1 : 0;
  a.la_pool = c->cfg.lookahead_pool;
  a.page_cluster = c->Nc > 0 ? c->d_page_cluster + lu * c->NP : nullptr;
  a.score_stride = c->Nc > 0 ? c->Nc : c->NP;
  a.page_bytes = (unsigned)c->page_bytes;
  return a;
}

hipError_t kvd_launch_select_resolve(kvd_ctx* c, int layer, int step, bool do_select, bool do_resolve, bool do_gather,
                                     const float* scores, int32_t* sel_pages, int32_t* sel_slots, int32_t* hit_mask,
                                     int32_t* evicted, int32_t* counts, int u0, int u1, hipStream_t s) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  const FastArgs a = kvd_fast_args(c, layer, step, do_gather, scores, sel_pages, sel_slots, hit_mask, evicted, counts, u0);
  const int ipt = (c->NP + kFastThreads - 1) / kFastThreads;
  if (do_select && do_resolve) launch_fast<true, true>(ipt, a, u1 - u0, s);
  else if (do_select) launch_fast<true, false>(ipt, a, u1 - u0, s);
  else launch_fast<false, true>(4, a, u1 - u0, s);
  return hipGetLastError();
}
