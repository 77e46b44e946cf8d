// The whole layer-step in one launch: score -> select -> resolve -> fetch -> attend -> merge, with
// the units of the layer pipelined through the stages individually (SFC Disaggregation taken to
// the granularity of one (sequence, KV head) unit: while one unit's pages are being selected or
// fetched, other units are being scored or attended).
//
// The grid is one-dimensional and ordered so that a workgroup depends only on workgroups with a
// lower index:
//     the scoring workgroups (`chunks` per unit) of units 0 .. lag-1;
//     then for every unit u: its selection workgroup, followed by the scoring workgroups of unit
//     u + lag (so that a selection workgroup is dispatched about when its scores are complete);
//     then for every unit u: its S attention workgroups.
// A selection workgroup waits until the unit's scoring workgroups have all arrived (a counter);
// an attention workgroup waits until the unit's selection, directory update and fetch are
// complete (a flag carrying the launch number).  Workgroups are dispatched in index order, so
// whatever a waiting workgroup waits for has already been dispatched and needs nothing from
// later workgroups: the lowest-numbered unfinished workgroup can always run to its end.  Every
// wait is nevertheless bounded by a wall-clock limit; a wait that runs out raises an error word in
// host memory and the workgroup leaves without output.
//
// Workgroups of one launch may sit on different XCDs with separate L2 caches.  Everything that
// crosses workgroups inside the launch (scores, the selection and its slots, fetched pages, split
// partials) is therefore written with device-scope write-through stores, and a flag is raised
// only after those stores have been acknowledged; flags, scores, the selection and the partials
// are read with device-scope loads.  Fetched pages are read with ordinary loads: no workgroup of
// the launch touches a slot before the flag of its unit is up, so no cache can hold an older copy.
#include "kvd_attn_body.h"
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_score_body.h"
#include "kvd_selres_body.h"

namespace kvd {

constexpr int kStepThreads = 512;
constexpr int kStepWaves = kStepThreads / kWave;

struct StepArgs {
  const uint16_t* summ;      // [U][NP][D] of the layer
  const uint16_t* q;         // [B][Hq][D]
  float* scores;             // [U][NP]
  FastArgs fa;
  AttnArgs at;
  int32_t* score_done;       // [U] scoring workgroups of the unit that have arrived; zero between launches
  int32_t* sel_ready;        // [U] number of the last launch whose selection for the unit is complete
  int32_t* error;            // host-visible; set when a wait runs out
  long long* timeline;       // [workgroups][5]: wall-clock ticks at start, wait over, work done, exit; then a tag; or null
  long long wait_limit;      // ticks of the 100 MHz wall clock
  float scale;
  int epoch, n_units, u0, chunks, passes, lag;
};

typedef AttnSmem<KVD_MAX_GROUP, kStepWaves> StepAttnSmem;
typedef FastSmem<kStepThreads> StepFastSmem;
constexpr size_t kStepSmemBytes = sizeof(StepAttnSmem) > sizeof(StepFastSmem) ? sizeof(StepAttnSmem) : sizeof(StepFastSmem);

template <bool BF16, int IPT>
__device__ __forceinline__ void step_body(const StepArgs& a, unsigned char* smem_raw, int& wait_ok) {
  const int tid = threadIdx.x;
  const int bid = blockIdx.x;
  long long* ts = a.timeline != nullptr && tid == 0 ? a.timeline + (size_t)bid * 5 : nullptr;
  if (ts) ts[0] = ts[1] = wall_clock64();
  const int per_unit = a.chunks + 1;
  const int front = a.n_units * per_unit;
  if (bid < front) {
    // front order: scoring of units 0..lag-1; then, for every unit u, its selection workgroup
    // followed by the scoring workgroups of unit u + lag
    int u, r;                                          // r < chunks: scoring workgroup r; r == chunks: selection
    const int lead = a.lag * a.chunks;
    if (bid < lead) {
      u = bid / a.chunks;
      r = bid % a.chunks;
    } else {
      const int j = bid - lead;
      const int n_full = a.n_units - a.lag;            // units whose selection is followed by a later unit's scoring
      if (j < n_full * per_unit) {
        const int g = j / per_unit, rr = j % per_unit;
        u = rr == 0 ? g : g + a.lag;
        r = rr == 0 ? a.chunks : rr - 1;
      } else {
        u = n_full + (j - n_full * per_unit);
        r = a.chunks;
      }
    }
    u += a.u0;
    if (ts) ts[4] = (r < a.chunks ? 0LL : 1LL) | ((long long)u << 8) | ((long long)(r < a.chunks ? r : 0) << 32);
    if (r < a.chunks) {
      // ---- scoring workgroup r of unit u
      const int b = u / a.fa.Hkv, h = u % a.fa.Hkv;
      const int w = tid / kWave;
      const int wave_base = (r * kStepWaves + w) * 64 * a.passes;
      score_wave<BF16, true>(a.summ + (size_t)u * a.fa.NP * kHeadDim,
                             a.q + ((size_t)b * a.at.Hq + (size_t)h * a.at.G) * kHeadDim, a.scores + (size_t)u * a.fa.NP,
                             a.fa.NP, a.at.G, a.scale, wave_base, a.passes);
      if (ts) ts[2] = wall_clock64();
      wave_drain_memory();                             // this wave's scores have been acknowledged
      __syncthreads();
      if (tid == 0) __hip_atomic_fetch_add(&a.score_done[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ts) ts[3] = wall_clock64();
      return;
    }
    // ---- selection, directory update and fetch of unit u: latency-bound, so its waves go first
    // whenever they can issue
    __builtin_amdgcn_s_setprio(3);
    if (!block_wait_equal(&a.score_done[u], a.chunks, a.wait_limit, &wait_ok)) {
      if (tid == 0) __hip_atomic_store(a.error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      return;
    }
    if (ts) ts[1] = wall_clock64();
    if (tid == 0) store_agent(&a.score_done[u], 0);    // every arrival has been seen: ready for the next launch
    StepFastSmem& sm = *reinterpret_cast<StepFastSmem*>(smem_raw);
    select_resolve_body<kStepThreads, IPT, true, true, true>(a.fa, u, sm);
    if (ts) ts[2] = wall_clock64();
    wave_drain_memory();                               // selection, slots and fetched pages have been written through
    __syncthreads();
    if (tid == 0) store_agent(&a.sel_ready[u], a.epoch);
    if (ts) ts[3] = wall_clock64();
    return;
  }
  // ---- attention workgroup (u, split)
  const int i = bid - front;
  const int u = i / a.at.S + a.u0, split = i % a.at.S;
  if (ts) ts[4] = 2LL | ((long long)u << 8) | ((long long)split << 32);
  if (!block_wait_equal(&a.sel_ready[u], a.epoch, a.wait_limit, &wait_ok)) {
    if (tid == 0) __hip_atomic_store(a.error, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return;
  }
  if (ts) ts[1] = wall_clock64();
  StepAttnSmem& sm = *reinterpret_cast<StepAttnSmem*>(smem_raw);
  attend_mfma_body<BF16, 0, kStepThreads, true, true>(a.at, sm, u, split);
  if (ts) ts[2] = ts[3] = wall_clock64();
}

template <bool BF16, int IPT>
__global__ __launch_bounds__(kStepThreads, 4) void step_kernel(StepArgs a) {
  __shared__ __align__(16) unsigned char smem_raw[kStepSmemBytes];
  __shared__ int wait_ok;
  step_body<BF16, IPT>(a, smem_raw, wait_ok);
}
template <bool BF16>
static void launch_step(int ipt, const StepArgs& a, int n_blocks, hipStream_t s) {
  dim3 grid(n_blocks), block(kStepThreads);
  if (ipt <= 8)
    hipLaunchKernelGGL((step_kernel<BF16, 8>), grid, block, 0, s, a);
  else if (ipt <= 16)
    hipLaunchKernelGGL((step_kernel<BF16, 16>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((step_kernel<BF16, 32>), grid, block, 0, s, a);
}

}  // namespace kvd

bool kvd_single_launch_ok(const kvd_ctx* c) {
  return kvd_fast_path_ok(c) && c->tiled && c->NP <= kvd::kStepThreads * 32;
}

hipError_t kvd_launch_step(kvd_ctx* c, int layer, int step, const void* q, float* out, float* lse, hipStream_t s) {
  using namespace kvd;
  StepArgs a;
  a.summ = reinterpret_cast<const uint16_t*>(c->summaries) + (size_t)layer * c->U * c->NP * kHeadDim;
  a.q = reinterpret_cast<const uint16_t*>(q);
  a.scores = c->d_scores;
  a.fa = kvd_fast_args(c, layer, step, true, c->d_scores, c->d_sel_pages, c->d_sel_slots, c->d_hit_mask, c->d_evicted,
                       c->d_counts, 0);
  a.at = kvd_attn_args(c, layer, q, c->d_sel_pages, c->d_sel_slots, out, lse, 0);
  a.at.fuse_merge = 1;
  a.score_done = c->d_score_done;
  a.sel_ready = c->d_sel_ready;
  a.error = c->error_dev;
  a.timeline = nullptr;
  a.wait_limit = c->wait_limit_ticks;
  a.scale = c->scale;
  if (++c->epoch <= 0) c->epoch = 1;
  a.epoch = c->epoch;
  a.n_units = c->U;
  a.u0 = 0;
  // scoring workgroups: 8 waves x 64 pages x passes each, about 1024 of them over the layer
  const long long pages = (long long)c->NP * c->U;
  int passes = (int)((pages + 512LL * 1024 / 2) / (512LL * 1024));
  if (passes < 1) passes = 1;
  a.passes = passes;
  a.chunks = (c->NP + 512 * passes - 1) / (512 * passes);
  // a unit's selection workgroup is dispatched `lag` units of scoring later than its own scoring:
  // about one round of resident workgroups (2 per CU), so that it finds its scores complete
  a.lag = 512 / a.chunks;
  if (a.lag < 1) a.lag = 1;
  if (a.lag > c->U) a.lag = c->U;
  const int n_blocks = c->U * (a.chunks + 1) + c->U * c->S;
  c->tl_workgroups = n_blocks;
  if (c->profiling == 2 && n_blocks <= KVD_TIMELINE_MAX) a.timeline = c->d_timeline;
  const int ipt = (c->NP + kStepThreads - 1) / kStepThreads;
  if (c->bf16) launch_step<true>(ipt, a, n_blocks, s);
  else launch_step<false>(ipt, a, n_blocks, s);
  return hipGetLastError();
}
