// The whole layer-step in one launch: score -> select -> resolve -> fetch -> attend -> merge, with
// the units of the layer pipelined through the stages individually (SFC Disaggregation taken to
// the granularity of one (sequence, KV head) unit: while one unit's pages are being selected or
// fetched, other units are being scored or attended).
//
// The grid is one-dimensional and ordered so that a workgroup depends only on workgroups with a
// lower index:
//     n_score persistent scoring workgroups, which take the layer's scoring chunks in turn, unit
//     by unit, so that the units' scores complete a round of scoring workgroups at a time, in unit
//     order, while scoring goes on;
//     then one selection workgroup per unit (with the hierarchical index it scores nothing itself:
//     the scoring workgroups score the centroids and it expands the best clusters into pages);
//     then S attention workgroups per unit.
// A launch may cover several consecutive layers of one decode step (kvd_step_layers, for a caller
// that has all their queries at hand).  The layers' blocks are then interleaved so that in-order
// dispatch pipelines the layers through the compute units:
//     score(0) select(0) | score(1) select(1) attend(0) | score(2) select(2) attend(1) | ... | attend(n-1)
// — the scoring of layer l+1 streams while layer l's units are being selected (and their missed
// pages fetched), and layer l's attention streams while layer l+1 is selected.  Every layer of the
// launch has its own directory, slots and set of per-step scratch; dependencies stay inside a layer
// and point to lower block indices only.
// The units of one layer can likewise be cut into groups that follow each other through the launch in
// the same interleaved order (SFC Disaggregation's micro-batches, pipelined by dispatch order instead
// of by streams): groups of one layer share the layer's scratch set, since all of it is indexed by unit.
// A selection workgroup waits until the unit's scoring waves have all arrived (a counter);
// an attention workgroup waits until the entries of its split have been published by the unit's
// selection workgroup (one word per selected page, published when the page is in its slot and
// blanked again by the unit's last attention workgroup).  Workgroups are
// dispatched in index order, so whatever a waiting workgroup waits for has already been dispatched
// and needs nothing from later workgroups: the lowest-numbered unfinished workgroup can always run
// to its end.  Every wait is nevertheless bounded by a wall-clock limit; a wait that runs out
// raises an error word in host memory and the workgroup leaves without output.
//
// Workgroups of one launch may sit on different XCDs with separate L2 caches.  Everything that
// crosses workgroups inside the launch (scores, the selection and its slots, fetched pages, split
// partials) is therefore written with device-scope write-through stores, and a counter is raised
// or an entry published only after those stores have been acknowledged; counters, scores, the
// entries and the partials are read with device-scope loads.  Fetched pages are read with
// ordinary loads: no workgroup of the launch touches a slot before the page's entry has been
// published, so no cache can hold an older copy.
#include "kvd_attn_body.h"
#include "kvd_cluster_body.h"
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_score_body.h"
#include "kvd_selres_body.h"

namespace kvd {

// One workgroup per CU in both forms:
constexpr int kStepThreads = 512;            // 256 registers per lane: three tile buffers in the attention role
constexpr int kStepThreadsWide = 1024;       // 128 registers per lane: units of more pages than 512 threads keep in registers

constexpr int kStepMaxLayers = KVD_MAX_SETS;   // layers one launch can cover: each needs a set of per-step scratch

// The per-step scratch of one layer of the launch.
struct StepLayerSet {
  float* scores;
  int32_t *sel_pages, *sel_slots, *hit_mask, *evicted, *counts, *miss_list, *miss_count;
  float *part_acc, *part_ml;
  int32_t *attn_ticket, *score_done;
  u64* sel_entry;
};

// The fields outside `sets` and the strides describe layer 0 of the launch; layer i of the launch
// (context layer layer0 + i) is found `i` strides further and works in sets[i].
struct StepArgs {
  const uint16_t* summ;      // [U][score_np][D] of the layer: the page summaries, or the centroids of the hierarchical index
  const uint16_t* q;         // [B][Hq][D]
  float* scores;             // [U][score_np]
  const int32_t* cluster_start;  // [U][Nc+1] of the layer, hierarchical index only
  const int32_t* cluster_pages;  // [U][NP]
  FastArgs fa;
  AttnArgs at;
  int32_t* score_done;       // [U][32] (one line per unit) scoring waves of the unit that have arrived (one per wave of the workgroup and chunk); zero between launches
  int32_t* error;            // host-visible; set when a wait runs out
  long long* timeline;       // [workgroups][5]: wall-clock ticks at start, wait over, work done, exit; then a tag; or null
  long long wait_limit;      // ticks of the 100 MHz wall clock
  float scale;
  int n_units, u0, chunks, passes, n_score;
  int score_np;              // rows scored per unit: NP, or the number of centroids Nc
  int Nc;                    // 0 = flat page index
  int n_layers;              // layers covered by the launch
  int groups, group_units;   // the units of a layer go through the launch in `groups` groups of group_units units (the last may be smaller)
  int layer0, Lp;            // first context layer; layers of the host store (layer l reads store layer l % Lp)
  const char* store_base;    // host store, layer 0 (device-visible address)
  long long summ_stride, q_stride, out_stride, lse_stride;           // elements between consecutive layers
  long long cluster_start_stride, cluster_pages_stride;              // elements
  long long pool_stride, store_stride;                               // bytes
  long long dir_unit_stride, dir_slot_stride, dir_page_stride;       // elements: [U], [U][Cmax] and [U][NP] tables
  StepLayerSet sets[kStepMaxLayers];
};

template <int NT>
struct StepSmem {
  typedef AttnSmem<KVD_MAX_GROUP, NT / kWave> Attn;
  typedef FastSmem<NT> Fast;
  typedef ClusterSelectSmem<NT> Cluster;               // behind Fast: a selection workgroup of the hierarchical index uses both at once
  static constexpr size_t cluster_at = (sizeof(Fast) + 15) & ~(size_t)15;
  static constexpr size_t bytes_fc = cluster_at + sizeof(Cluster);
  static constexpr size_t bytes = sizeof(Attn) > bytes_fc ? sizeof(Attn) : bytes_fc;
};

// The three roles read the launch arguments from the kernel-argument segment (constant address
// space, scalar loads) and copy only what they use.
typedef const __attribute__((address_space(4))) StepArgs* StepArgsPtr;
constexpr int kFlagStride = 32;   // ints between the flags of two units: one 128-byte line each

// Scoring workgroup `wg` of n_score: chunks wg, wg + n_score, ... of the layer, unit by unit.
// A unit's selection workgroup waits for chunks * (NT / 64) arrivals, one per scoring wave and
// chunk.  Arrivals at one address from all over the chip are slow (a few tens of nanoseconds each,
// one after the other), so the waves of a workgroup first count themselves in LDS and the last of
// them to finish a chunk reports all of them with one add; a workgroup's chunks past kScoreSlots
// fall back to one add per wave.
constexpr int kScoreSlots = 32;                       // (the configurations of the benchmark take 2 to 5 chunks per workgroup)
template <bool BF16, int NT>
__device__ __forceinline__ void step_score_role(StepArgsPtr ap, int li, int u0, int n_units, int wg, unsigned char* smem_raw,
                                                long long* ts) {
  struct { const uint16_t* summ; const uint16_t* q; float* scores; int32_t* score_done; float scale;
           int n_units, chunks, n_score, u0, passes; struct { int Hkv, NP; } fa; struct { int Hq, G; } at; } a;   // (fa.NP: rows scored per unit)
  a.summ = ap->summ + (long long)li * ap->summ_stride; a.q = ap->q + (long long)li * ap->q_stride;
  a.scores = ap->sets[li].scores; a.score_done = ap->sets[li].score_done; a.scale = ap->scale;
  a.n_units = n_units; a.chunks = ap->chunks; a.n_score = ap->n_score; a.u0 = u0; a.passes = ap->passes;
  a.fa.Hkv = ap->fa.Hkv; a.fa.NP = ap->score_np; a.at.Hq = ap->at.Hq; a.at.G = ap->at.G;
  const int tid = threadIdx.x;
  const int w = tid / kWave, lane = tid & (kWave - 1);
  if (ts) ts[4] = 0LL | ((long long)wg << 32);
  int* arrived = reinterpret_cast<int*>(smem_raw);     // [kScoreSlots] waves of this workgroup done with its i-th chunk
  for (int i = tid; i < kScoreSlots; i += NT) arrived[i] = 0;
  __syncthreads();
  const int total = a.n_units * a.chunks;
  int ordinal = 0;
  for (int c = wg; c < total; c += a.n_score, ++ordinal) {
    const int u = c / a.chunks + a.u0, r = c % a.chunks;
    const int b = u / a.fa.Hkv, h = u % a.fa.Hkv;
    const int wave_base = (r * (NT / kWave) + w) * 64 * a.passes;
    score_wave<BF16, true>(a.summ + (size_t)u * a.fa.NP * kHeadDim,
                           a.q + ((size_t)b * a.at.Hq + (size_t)h * a.at.G) * kHeadDim, a.scores + (size_t)u * a.fa.NP,
                           a.fa.NP, a.at.G, a.scale, wave_base, a.passes);
    wave_drain_memory();                               // this wave's scores have been acknowledged
    if (lane == 0) {
      int add = 1;
      if (ordinal < kScoreSlots)
        add = __hip_atomic_fetch_add(&arrived[ordinal], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP) == NT / kWave - 1 ? NT / kWave : 0;
      if (add) __hip_atomic_fetch_add(&a.score_done[u * kFlagStride], add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (ts) ts[2] = ts[3] = wall_clock64();
}

// Selection, directory update and fetch of unit u: latency-bound, so its waves go first whenever
// they can issue.
template <int NT, int IPT>
__device__ __forceinline__ void step_select_role(StepArgsPtr ap, int li, int u, unsigned char* smem_raw, int* wait_ok,
                                                           long long* ts) {
  struct { FastArgs fa; int32_t* score_done; int32_t* error; long long wait_limit; int chunks; } a;
  __builtin_memcpy(&a.fa, &ap->fa, sizeof(FastArgs));
  {
    // this layer's directory, slots, stored pages and scratch
    const long long l = li;
    a.fa.capacity += l * ap->dir_unit_stride;
    a.fa.resident += l * ap->dir_unit_stride;
    a.fa.slot_page += l * ap->dir_slot_stride;
    a.fa.slot_stamp += l * ap->dir_slot_stride;
    if (a.fa.page_cluster != nullptr) a.fa.page_cluster += l * ap->dir_page_stride;
    a.fa.pool += l * ap->pool_stride;
    a.fa.store = ap->store_base + (long long)((ap->layer0 + li) % ap->Lp) * ap->store_stride;
    a.fa.scores = ap->sets[li].scores; a.fa.sel_pages = ap->sets[li].sel_pages; a.fa.sel_slots = ap->sets[li].sel_slots;
    a.fa.sel_entry = ap->sets[li].sel_entry; a.fa.hit_mask = ap->sets[li].hit_mask; a.fa.evicted = ap->sets[li].evicted;
    a.fa.counts = ap->sets[li].counts; a.fa.miss_list = ap->sets[li].miss_list; a.fa.miss_count = ap->sets[li].miss_count;
  }
  a.score_done = ap->sets[li].score_done; a.error = ap->error;
  a.wait_limit = ap->wait_limit; a.chunks = ap->chunks;
  const int tid = threadIdx.x;
  if (ts) ts[4] = 1LL | ((long long)u << 8);
  __builtin_amdgcn_s_setprio(3);
  typename StepSmem<NT>::Fast& sm = *reinterpret_cast<typename StepSmem<NT>::Fast*>(smem_raw);
  // the directory is loaded and the LDS tables are set up while the unit's scores are still coming in
  auto scores_ready = [&]() -> bool {
    const bool ok = block_wait_equal(&a.score_done[u * kFlagStride], a.chunks * (NT / kWave), a.wait_limit, wait_ok);
    if (ts) ts[1] = wall_clock64();
    if (ok && tid == 0) store_agent(&a.score_done[u * kFlagStride], 0);   // every arrival has been seen: ready for the next launch
    return ok;
  };
  bool done;
  if (ap->Nc > 0) {
    // hierarchical index: the scores are those of the centroids.  The directory update's loads and
    // LDS tables and the cluster bounds are under way while the unit's scores are still coming in;
    // once they are there the clusters are expanded into pages, which reach the directory update
    // through LDS.
    typename StepSmem<NT>::Cluster& cs = *reinterpret_cast<typename StepSmem<NT>::Cluster*>(smem_raw + StepSmem<NT>::cluster_at);
    const int32_t* cstart = ap->cluster_start + (long long)li * ap->cluster_start_stride;
    const int32_t* cpages = ap->cluster_pages + (long long)li * ap->cluster_pages_stride;
    const int Nc = ap->Nc;
    auto select_clusters = [&]() -> bool {
      ClusterPrep<NT> prep;
      cluster_prepare<NT>(cstart, cpages, a.fa.seq_len, a.fa.NP, Nc, a.fa.P, a.fa.k, a.fa.sink, a.fa.recent, a.fa.Hkv, u, prep);
      if (!scores_ready()) return false;
      cluster_finish<NT, true>(a.fa.scores, cpages, a.fa.sel_pages, sm.sel, a.fa.NP, Nc, a.fa.k, u, prep, cs);
      __syncthreads();                                 // the selection is complete
      return true;
    };
    done = select_resolve_body<NT, 4, false, true, true, decltype(select_clusters), true>(a.fa, u, sm, select_clusters);
  } else {
    done = select_resolve_body<NT, IPT, true, true, true>(a.fa, u, sm, scores_ready);
  }
  if (!done) {
    if (tid == 0) __hip_atomic_store(a.error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    return;
  }
  if (ts) ts[2] = ts[3] = wall_clock64();              // (the entries have been published inside)
}

// Attention workgroup (u, split).
template <bool BF16, int NT, bool LEAN, bool PACKED>
__device__ __forceinline__ void step_attend_role(StepArgsPtr ap, int li, int u, int split, unsigned char* smem_raw, long long* ts) {
  struct { AttnArgs at; } a;
  __builtin_memcpy(&a.at, &ap->at, sizeof(AttnArgs));
  {
    const long long l = li;
    a.at.q += l * ap->q_stride;
    a.at.pool += l * ap->pool_stride;
    a.at.out += l * ap->out_stride;
    if (a.at.lse != nullptr) a.at.lse += l * ap->lse_stride;
    a.at.sel_pages = ap->sets[li].sel_pages; a.at.sel_slots = ap->sets[li].sel_slots; a.at.sel_entry = ap->sets[li].sel_entry;
    a.at.part_acc = ap->sets[li].part_acc; a.at.part_ml = ap->sets[li].part_ml; a.at.ticket = ap->sets[li].attn_ticket;
  }
  if (ts) ts[4] = 2LL | ((long long)u << 8) | ((long long)split << 32);
  typename StepSmem<NT>::Attn& sm = *reinterpret_cast<typename StepSmem<NT>::Attn*>(smem_raw);
  const int done = attend_mfma_body<BF16, 0, NT, true, LEAN, PACKED>(a.at, sm, u, split, ts ? ts + 1 : nullptr);
  if (done < 0 && threadIdx.x == 0) __hip_atomic_store(a.at.error, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  if (ts) ts[2] = ts[3] = wall_clock64();
}

template <bool BF16, int NT, int IPT, bool LEAN, bool PACKED>
__device__ __forceinline__ void step_body(StepArgsPtr ap, unsigned char* smem_raw, int& wait_ok) {
  const int bid = blockIdx.x;
  long long* timeline = ap->timeline;
  long long* ts = timeline != nullptr && threadIdx.x == 0 ? timeline + (size_t)bid * 5 : nullptr;
  if (ts) { ts[0] = ts[1] = ts[2] = ts[3] = wall_clock64(); ts[4] = 3LL; }   // (role 3: a workgroup beyond its group's units, which leaves at once)
  const int n_score = ap->n_score, S = ap->at.S, groups = ap->groups, Ug = ap->group_units;
  const int n_stages = ap->n_layers * groups;          // (layer, group) pairs, in order
  const int front = n_score + Ug, back = Ug * S;
  // block order: front(0) | front(1) back(0) | front(2) back(1) | ... | back(n-1), where front(i) =
  // the scoring and selection workgroups of stage i and back(i) its attention workgroups
  int st = 0, o = bid;
  bool is_back = false;
  if (bid >= front) {
    const int r = bid - front, per = front + back;
    const int g = r / per;
    o = r % per;
    if (g < n_stages - 1) {
      if (o < front) { st = g + 1; } else { st = g; o -= front; is_back = true; }
    } else {
      st = n_stages - 1; is_back = true;
    }
  }
  const int li = st / groups, u0 = ap->u0 + (st % groups) * Ug;
  int n_units = ap->n_units - (st % groups) * Ug;       // units of this group
  n_units = n_units < Ug ? n_units : Ug;
  if (is_back) {
    if (o / S < n_units) step_attend_role<BF16, NT, LEAN, PACKED>(ap, li, o / S + u0, o % S, smem_raw, ts);
  } else if (o < n_score) {
    step_score_role<BF16, NT>(ap, li, u0, n_units, o, smem_raw, ts);
  } else {
    if (o - n_score < n_units) step_select_role<NT, IPT>(ap, li, o - n_score + u0, smem_raw, &wait_ok, ts);
  }
}

// LEAN: 128 registers per lane (the 1024-thread form); otherwise 256.  PACKED: pages of 4 or 8 tokens.
template <bool BF16, int NT, int IPT, bool PACKED, bool LEAN = (NT > kStepThreads)>
__global__ __launch_bounds__(NT, LEAN ? 4 : 2) void step_kernel(StepArgs a) {
  __shared__ __align__(16) unsigned char smem_raw[StepSmem<NT>::bytes];
  __shared__ int wait_ok;
  // the launch arguments are the first thing in the kernel-argument segment
  step_body<BF16, NT, IPT, LEAN, PACKED>((StepArgsPtr)__builtin_amdgcn_kernarg_segment_ptr(), smem_raw, wait_ok);
}
template <bool BF16, bool PACKED>
static void launch_step(int threads, int ipt, const StepArgs& a, int n_blocks, hipStream_t s) {
  dim3 grid(n_blocks), block(threads);
  if (threads == kStepThreadsWide) {
    if (ipt <= 8)
      hipLaunchKernelGGL((step_kernel<BF16, kStepThreadsWide, 8, PACKED>), grid, block, 0, s, a);
    else
      hipLaunchKernelGGL((step_kernel<BF16, kStepThreadsWide, 16, PACKED>), grid, block, 0, s, a);
  } else if (ipt <= 4) {
    hipLaunchKernelGGL((step_kernel<BF16, kStepThreads, 4, PACKED>), grid, block, 0, s, a);
  } else if (ipt <= 8) {
    hipLaunchKernelGGL((step_kernel<BF16, kStepThreads, 8, PACKED>), grid, block, 0, s, a);
  } else {
    hipLaunchKernelGGL((step_kernel<BF16, kStepThreads, 16, PACKED>), grid, block, 0, s, a);
  }
}

}  // namespace kvd

// The launch shape of the one-launch step.  What kvd_set_step_shape / kvd_calibrate_step_shape fixed
// is taken; the rest follows the rule: one group; scoring workgroups = one round of resident
// workgroups (one per CU) minus 1/8 left to the selection workgroups that run beside them; passes
// such that the chunks of a group fill whole rounds of its scoring workgroups (time ~ rounds x
// passes; at equal cost the coarser chunk wins while every scoring workgroup still gets one: fewer
// reports and acknowledgement waits per byte); splits as kvd_create chose them.
kvd_shape kvd_step_shape(const kvd_ctx* c, int multi_layer, const kvd_shape* want) {
  kvd_shape w = want ? *want : c->shape[multi_layer ? 1 : 0];
  const int score_np = c->Nc > 0 ? c->Nc : c->NP;
  const int chunk_pages = c->step_threads == kvd::kStepThreadsWide ? kvd::kStepThreadsWide : kvd::kStepThreads;
  const int slots = c->n_cus;
  kvd_shape e;
  e.groups = w.groups > 0 ? w.groups : 1;
  if (e.groups > c->U) e.groups = c->U;
  const int Ug = (c->U + e.groups - 1) / e.groups;      // units per group
  e.groups = (c->U + Ug - 1) / Ug;                      // (no empty group)
  int ns = w.n_score;
  if (ns <= 0) {
    int reserve = slots / 8;
    if (reserve > Ug) reserve = Ug;
    ns = slots - reserve;
  }
  if (ns < 1) ns = 1;
  int ps = w.passes;
  if (ps <= 0) {
    long long best_cost = -1;
    for (int cand = 1; cand <= 8; ++cand) {
      const long long chunks = (score_np + (long long)chunk_pages * cand - 1) / ((long long)chunk_pages * cand);
      const long long rounds = (chunks * Ug + ns - 1) / ns;
      const long long cost = rounds * cand;
      if (best_cost < 0 || cost < best_cost || (cost == best_cost && chunks * Ug >= ns)) { best_cost = cost; ps = cand; }
    }
  }
  const int chunks = (score_np + chunk_pages * ps - 1) / (chunk_pages * ps);
  if (ns > Ug * chunks) ns = Ug * chunks;
  e.passes = ps;
  e.n_score = ns;
  e.splits = w.splits > 0 ? w.splits : c->S1;
  return e;
}

// Which shapes the context can run: passes 1..8; 1..(compute units) scoring workgroups; splits
// within what the partials were allocated for, with a split's entries fitting their LDS staging
// area; 1..8 groups.
bool kvd_step_shape_ok(const kvd_ctx* c, const kvd_shape& e) {
  if (e.passes < 1 || e.passes > 8 || e.n_score < 1 || e.n_score > c->n_cus) return false;
  if (e.splits < 1 || e.splits > c->S1_max || e.splits > c->k) return false;
  if ((c->k + e.splits - 1) / e.splits > kvd::kAttnIdxCap) return false;
  if (e.groups < 1 || e.groups > 8) return false;
  return true;
}

bool kvd_single_launch_ok(const kvd_ctx* c) {
  return kvd_fast_path_ok(c) && c->tiled && c->NP <= kvd::kStepThreadsWide * 16 &&
         (c->k + c->S1 - 1) / c->S1 <= kvd::kAttnIdxCap;   // a split's entries are staged in LDS
}

hipError_t kvd_launch_step(kvd_ctx* c, int layer, int n_layers, int step, const void* q, float* out, float* lse, hipStream_t s) {
  using namespace kvd;
  if (n_layers < 1 || n_layers > kStepMaxLayers || n_layers > c->n_sets || layer + n_layers > c->L) return hipErrorInvalidValue;
  StepArgs a;
  const int score_np = c->Nc > 0 ? c->Nc : c->NP;
  a.summ = reinterpret_cast<const uint16_t*>(c->Nc > 0 ? c->centroids : c->summaries) + (size_t)layer * c->U * score_np * kHeadDim;
  a.score_np = score_np;
  a.Nc = c->Nc;
  a.cluster_start = c->Nc > 0 ? c->cluster_start + (size_t)layer * c->U * (c->Nc + 1) : nullptr;
  a.cluster_pages = c->Nc > 0 ? c->cluster_pages + (size_t)layer * c->U * c->NP : nullptr;
  a.q = reinterpret_cast<const uint16_t*>(q);
  a.scores = c->d_scores;
  a.fa = kvd_fast_args(c, layer, step, true, c->d_scores, c->d_sel_pages, c->d_sel_slots, c->d_hit_mask, c->d_evicted,
                       c->d_counts, 0);
  a.at = kvd_attn_args(c, layer, q, c->d_sel_pages, c->d_sel_slots, out, lse, 0);
  a.at.fuse_merge = 1;
  a.at.sel_entry = c->d_sel_entry;
  const kvd_shape shape = kvd_step_shape(c, n_layers > 1);
  a.at.S = shape.splits;
  a.at.per_split = (c->k + shape.splits - 1) / shape.splits;
  a.score_done = c->d_score_done;
  a.error = c->error_dev;
  a.timeline = nullptr;
  a.wait_limit = c->wait_limit_ticks;
  a.scale = c->scale;
  a.n_units = c->U;
  a.u0 = 0;
  // the layers of the launch: layer `layer + i` works in scratch set i
  a.n_layers = n_layers;
  a.layer0 = layer;
  a.Lp = c->Lp;
  a.store_base = c->store_dev;
  a.summ_stride = (long long)c->U * score_np * kHeadDim;
  a.q_stride = (long long)c->B * c->Hq * kHeadDim;
  a.out_stride = (long long)c->B * c->Hq * kHeadDim;
  a.lse_stride = (long long)c->B * c->Hq;
  a.cluster_start_stride = (long long)c->U * (c->Nc + 1);
  a.cluster_pages_stride = (long long)c->U * c->NP;
  a.pool_stride = (long long)c->U * c->Cmax * (long long)c->page_bytes;
  a.store_stride = (long long)c->U * c->NP * (long long)c->page_bytes;
  a.dir_unit_stride = c->U;
  a.dir_slot_stride = (long long)c->U * c->Cmax;
  a.dir_page_stride = (long long)c->U * c->NP;
  for (int i = 0; i < kStepMaxLayers; ++i) {
    const kvd_scratch x = kvd_scratch_set(c, i < n_layers ? i : 0);
    StepLayerSet& d = a.sets[i];
    d.scores = x.scores; d.sel_pages = x.sel_pages; d.sel_slots = x.sel_slots; d.hit_mask = x.hit_mask; d.evicted = x.evicted;
    d.counts = x.counts; d.miss_list = x.miss_list; d.miss_count = x.miss_count; d.part_acc = x.part_acc; d.part_ml = x.part_ml;
    d.attn_ticket = x.attn_ticket; d.score_done = x.score_done; d.sel_entry = x.sel_entry;
  }
  if (n_layers == 1) {
    // (a single layer works in the context's current set, whichever that is)
    StepLayerSet& d = a.sets[0];
    d.scores = c->d_scores; d.sel_pages = c->d_sel_pages; d.sel_slots = c->d_sel_slots; d.hit_mask = c->d_hit_mask;
    d.evicted = c->d_evicted; d.counts = c->d_counts; d.miss_list = c->d_miss_list; d.miss_count = c->d_miss_count;
    d.part_acc = c->d_part_acc; d.part_ml = c->d_part_ml; d.attn_ticket = c->d_attn_ticket; d.score_done = c->d_score_done;
    d.sel_entry = c->d_sel_entry;
  }
  // Units of more than 8192 pages take the 1024-thread form, whose selection role keeps at most
  // 16 pages per thread in registers like the 512-thread form does for the others.
  const int threads = c->step_threads == kStepThreadsWide ? kStepThreadsWide : kStepThreads;
  const int chunk_pages = threads;                    // a scoring chunk: every wave 64 pages x passes
  a.passes = shape.passes;
  a.n_score = shape.n_score;
  a.groups = shape.groups;
  a.group_units = (c->U + shape.groups - 1) / shape.groups;
  a.chunks = (score_np + chunk_pages * a.passes - 1) / (chunk_pages * a.passes);
  const int n_blocks = n_layers * a.groups * (a.n_score + a.group_units + a.group_units * shape.splits);
  c->tl_workgroups = n_blocks;
  if (c->profiling == 2 && n_blocks <= KVD_TIMELINE_MAX) a.timeline = c->d_timeline;
  const int ipt = (c->NP + chunk_pages - 1) / chunk_pages;
  const bool packed = c->tiled == kLayoutPacked;
  if (c->bf16) { if (packed) launch_step<true, true>(threads, ipt, a, n_blocks, s); else launch_step<true, false>(threads, ipt, a, n_blocks, s); }
  else { if (packed) launch_step<false, true>(threads, ipt, a, n_blocks, s); else launch_step<false, false>(threads, ipt, a, n_blocks, s); }
  return hipGetLastError();
}
