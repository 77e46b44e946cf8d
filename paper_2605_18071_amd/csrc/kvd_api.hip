// C ABI of libkvd: argument checks, the context, and the stream choreography of one layer-step.
// No stage is computed on the host; every hot-path entry point only enqueues kernels.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "kvd_internal.h"
#include "kvd_tile_layout.h"

#define KVD_ABI_VERSION 2

#define HIP_TRY(ctx, expr)                  \
  do {                                      \
    hipError_t _e = (expr);                 \
    if (_e != hipSuccess) {                 \
      if (ctx) (ctx)->last_hip = (int)_e;   \
      return KVD_ERR_HIP;                   \
    }                                       \
  } while (0)

// micro_batches -1 asks for the one-launch step wherever it can run; 0 leaves the choice to the
// library, which takes it where it has measured faster than the chain of kernels: everywhere in
// the 512-thread form (4 to 128 units measured, 2-6 us per step), and from 24 units on in the
// 1024-thread form (units of more than 8192 pages: 3-5 % slower than the chain with 8 and 16
// units, 18 % faster with 24).
static bool kvd_wants_single_launch(const kvd_ctx* c) {
  if (!kvd_single_launch_ok(c)) return false;
  if (c->cfg.micro_batches == -1) return true;
  return c->cfg.micro_batches == 0 && (c->step_threads != 1024 || c->U >= 24);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int validate_config(const kvd_config* c) {
  if (c == nullptr) return KVD_ERR_ARG;
  if (c->kv_dtype != KVD_F16 && c->kv_dtype != KVD_BF16) return KVD_ERR_DTYPE;
  if (c->policy != KVD_EVICT_LRU && c->policy != KVD_EVICT_LOOKAHEAD) return KVD_ERR_ARG;
  if (c->n_layers < 1 || c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return KVD_ERR_SHAPE;
  if (c->head_dim != 128) return KVD_ERR_SHAPE;
  if (c->n_q_heads % c->n_kv_heads != 0) return KVD_ERR_SHAPE;
  const int G = c->n_q_heads / c->n_kv_heads;
  if (G > KVD_MAX_GROUP) return KVD_ERR_SHAPE;
  if (c->page_size < 1 || c->page_size > KVD_MAX_PAGE) return KVD_ERR_SHAPE;
  if (c->max_pages < 1 || c->max_pages > (1 << 24)) return KVD_ERR_SHAPE;
  if (c->topk_pages < 1 || c->topk_pages > KVD_MAX_TOPK) return KVD_ERR_SHAPE;
  if (c->capacity_max < 1 || c->capacity_max > KVD_MAX_CAPACITY) return KVD_ERR_SHAPE;
  if ((long long)c->batch * c->n_kv_heads > 65535) return KVD_ERR_SHAPE;
  if (c->sink_pages < 0 || c->recent_pages < 0) return KVD_ERR_SHAPE;
  if (c->physical_layers < 0 || c->physical_layers > c->n_layers) return KVD_ERR_SHAPE;
  if (c->micro_batches < -1 || c->micro_batches > KVD_MAX_MICRO) return KVD_ERR_SHAPE;
  if (c->attn_splits < 0 || c->attn_splits > KVD_MAX_SPLITS) return KVD_ERR_SHAPE;
  if (c->index_centroids < 0 || c->index_centroids > KVD_MAX_CENTROIDS || c->index_centroids > c->max_pages) return KVD_ERR_SHAPE;
  if (c->index_centroids > 0 && c->max_pages > KVD_FAST_MAX_PAGES) return KVD_ERR_SHAPE;
  if (c->lookahead_pool < 0) return KVD_ERR_SHAPE;
  if (!(c->softmax_scale >= 0.f) || isinf(c->softmax_scale)) return KVD_ERR_ARG;
  if ((long long)c->sink_pages + c->recent_pages > c->topk_pages) return KVD_ERR_CAPACITY;
  if (c->topk_pages > c->capacity_max) return KVD_ERR_CAPACITY;
  if (c->capacity != nullptr) {
    const long long n = (long long)c->n_layers * c->batch * c->n_kv_heads;
    for (long long i = 0; i < n; ++i) {
      if (c->capacity[i] > c->capacity_max) return KVD_ERR_SHAPE;
      if (c->capacity[i] < c->topk_pages) return KVD_ERR_CAPACITY;
    }
  }
  return KVD_OK;
}

static void free_ctx(kvd_ctx* c) {
  if (c == nullptr) return;
  void* dev[] = {c->d_capacity, c->d_seq_len, c->d_page_to_slot, c->d_slot_page, c->d_slot_stamp, c->d_resident, c->d_page_cluster,
                 c->d_scores, c->d_sel_pages, c->d_sel_slots, c->d_hit_mask, c->d_evicted, c->d_counts,
                 c->d_miss_list, c->d_miss_count, c->d_part_acc, c->d_part_ml, c->d_attn_ticket, c->d_stats,
                 c->d_score_done, c->d_sel_entry, c->d_timeline};
  for (void* p : dev)
    if (p) (void)hipFree(p);
  for (int i = 0; i < c->n_sets; ++i) {
    if (i == c->cur_set) continue;                     // (that one is in the d_* fields)
    const kvd_scratch& x = c->sets[i];
    void* more[] = {x.scores, x.sel_pages, x.sel_slots, x.hit_mask, x.evicted, x.counts, x.miss_list, x.miss_count,
                    x.part_acc, x.part_ml, x.attn_ticket, x.score_done, x.sel_entry};
    for (void* p : more)
      if (p) (void)hipFree(p);
  }
  for (int i = 0; i < KVD_MAX_MICRO; ++i) {
    if (c->ev_score[i]) (void)hipEventDestroy(c->ev_score[i]);
    if (c->ev_done[i]) (void)hipEventDestroy(c->ev_done[i]);
  }
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  for (int i = 0; i < 12; ++i)
    if (c->ev_prof[i]) (void)hipEventDestroy(c->ev_prof[i]);
  for (int i = 0; i < KVD_PIPE_STREAMS; ++i)
    if (c->side[i]) (void)hipStreamDestroy(c->side[i]);
  if (c->error_host) (void)hipHostFree(c->error_host);
  if (c->h_miss_list) (void)hipHostFree(c->h_miss_list);
  if (c->h_miss_count) (void)hipHostFree(c->h_miss_count);
  if (c->h_src_offset) (void)hipHostFree(c->h_src_offset);
  if (c->d_src_offset) (void)hipFree(c->d_src_offset);
  free(c->h_capacity);
  free(c->h_seq_len);
  free(c);
}

// Side streams and events for a step in `groups` groups; created on first need, kept until destroy.
static hipError_t ensure_group_resources(kvd_ctx* c, int groups) {
  if (groups <= 1) return hipSuccess;
  for (int i = 0; i < KVD_PIPE_STREAMS; ++i)
    if (c->side[i] == nullptr) {
      const hipError_t e = hipStreamCreateWithFlags(&c->side[i], hipStreamNonBlocking);
      if (e != hipSuccess) return e;
    }
  for (int i = 0; i < groups && i < KVD_MAX_MICRO; ++i) {
    if (c->ev_score[i] == nullptr) {
      const hipError_t e = hipEventCreateWithFlags(&c->ev_score[i], hipEventDisableTiming);
      if (e != hipSuccess) return e;
    }
    if (c->ev_done[i] == nullptr) {
      const hipError_t e = hipEventCreateWithFlags(&c->ev_done[i], hipEventDisableTiming);
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

template <class T>
static hipError_t dev_alloc(T** p, size_t count) {
  return hipMalloc(reinterpret_cast<void**>(p), (count ? count : 1) * sizeof(T));
}

// Makes scratch set `set` the one in the context's d_* fields.  Kernel arguments are taken at
// launch, so launches already enqueued keep the set they were given.
static void use_scratch_set(kvd_ctx* c, int set) {
  if (set == c->cur_set) return;
  kvd_scratch& o = c->sets[c->cur_set];
  o.scores = c->d_scores; o.sel_pages = c->d_sel_pages; o.sel_slots = c->d_sel_slots; o.hit_mask = c->d_hit_mask;
  o.evicted = c->d_evicted; o.counts = c->d_counts; o.miss_list = c->d_miss_list; o.miss_count = c->d_miss_count;
  o.part_acc = c->d_part_acc; o.part_ml = c->d_part_ml; o.attn_ticket = c->d_attn_ticket; o.score_done = c->d_score_done;
  o.sel_entry = c->d_sel_entry;
  const kvd_scratch& x = c->sets[set];
  c->d_scores = x.scores; c->d_sel_pages = x.sel_pages; c->d_sel_slots = x.sel_slots; c->d_hit_mask = x.hit_mask;
  c->d_evicted = x.evicted; c->d_counts = x.counts; c->d_miss_list = x.miss_list; c->d_miss_count = x.miss_count;
  c->d_part_acc = x.part_acc; c->d_part_ml = x.part_ml; c->d_attn_ticket = x.attn_ticket; c->d_score_done = x.score_done;
  c->d_sel_entry = x.sel_entry;
  c->cur_set = set;
}

kvd_scratch kvd_scratch_set(const kvd_ctx* c, int i) {
  if (i != c->cur_set) return c->sets[i];
  kvd_scratch o;
  o.scores = c->d_scores; o.sel_pages = c->d_sel_pages; o.sel_slots = c->d_sel_slots; o.hit_mask = c->d_hit_mask;
  o.evicted = c->d_evicted; o.counts = c->d_counts; o.miss_list = c->d_miss_list; o.miss_count = c->d_miss_count;
  o.part_acc = c->d_part_acc; o.part_ml = c->d_part_ml; o.attn_ticket = c->d_attn_ticket; o.score_done = c->d_score_done;
  o.sel_entry = c->d_sel_entry;
  return o;
}

static int reset_directory(kvd_ctx* c, int layer_or_all) {
  const int l0 = layer_or_all < 0 ? 0 : layer_or_all;
  const int nl = layer_or_all < 0 ? c->L : 1;
  const size_t lu = (size_t)l0 * c->U, nu = (size_t)nl * c->U;
  if (c->d_page_to_slot) HIP_TRY(c, kvd_launch_fill_i32(c->d_page_to_slot + lu * c->NP, -1, nu * c->NP, nullptr));
  HIP_TRY(c, kvd_launch_fill_i32(c->d_slot_page + lu * c->Cmax, -1, nu * c->Cmax, nullptr));
  HIP_TRY(c, kvd_launch_fill_i32(c->d_slot_stamp + lu * c->Cmax, -1, nu * c->Cmax, nullptr));
  HIP_TRY(c, kvd_launch_fill_i32(c->d_resident + lu, 0, nu, nullptr));
  HIP_TRY(c, hipDeviceSynchronize());
  return KVD_OK;
}

// Zeroes the words through which the workgroups of a one-launch step synchronise (all scratch sets).
static int clear_step_flags(kvd_ctx* c) {
  HIP_TRY(c, hipMemset(c->d_attn_ticket, 0, (size_t)c->U * sizeof(int32_t)));
  HIP_TRY(c, hipMemset(c->d_score_done, 0, (size_t)c->U * 32 * sizeof(int32_t)));
  HIP_TRY(c, hipMemset(c->d_sel_entry, 0, (size_t)c->U * c->k * sizeof(unsigned long long)));
  for (int i = 0; i < c->n_sets; ++i) {
    if (i == c->cur_set) continue;
    HIP_TRY(c, hipMemset(c->sets[i].attn_ticket, 0, (size_t)c->U * sizeof(int32_t)));
    HIP_TRY(c, hipMemset(c->sets[i].score_done, 0, (size_t)c->U * 32 * sizeof(int32_t)));
    HIP_TRY(c, hipMemset(c->sets[i].sel_entry, 0, (size_t)c->U * c->k * sizeof(unsigned long long)));
  }
  return KVD_OK;
}

// An in-kernel wait of a one-launch step ran out (the error word is set): that step produced no
// output for the units concerned and may have left their directory half updated.  The library then
// takes itself out of harm's way: it waits for the device, empties every layer's window, clears
// the flags and the error word and switches the context to the chain of kernels, which has no
// waits between workgroups.  The caller is told once, by the status of the call that finds the
// error; later steps run (from a cold cache, as a chain).  Returns the status to hand back.
static int recover_from_wait_timeout(kvd_ctx* c) {
  HIP_TRY(c, hipDeviceSynchronize());
  int r = clear_step_flags(c);
  if (r != KVD_OK) return r;
  r = reset_directory(c, -1);
  if (r != KVD_OK) return r;
  *c->error_host = 0;
  ++c->wait_timeouts;
  c->cfg.micro_batches = 1;
  c->MB = 1;
  c->single_launch = 0;
  return KVD_ERR_STATE;
}

extern "C" {

int kvd_abi_version(void) { return KVD_ABI_VERSION; }

const char* kvd_strerror(int status) {
  switch (status) {
    case KVD_OK: return "ok";
    case KVD_ERR_ARG: return "bad argument (NULL, misaligned, out of range, or not addressable by the GPU)";
    case KVD_ERR_SHAPE: return "inconsistent or unsupported sizes";
    case KVD_ERR_CAPACITY: return "capacity too small (k > C, forced pages > k, warm list > C, or a step needs more extents than the tier's pool holds)";
    case KVD_ERR_DTYPE: return "unsupported KV dtype";
    case KVD_ERR_HIP: return "HIP runtime call failed (see kvd_last_hip_error)";
    case KVD_ERR_STATE: return "buffers not bound, directory invariants violated, an in-kernel wait ran out, or a file operation of the tier failed";
    default: return "unknown status";
  }
}

int kvd_last_hip_error(const kvd_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int kvd_create(const kvd_config* cfg, kvd_ctx** out) {
  if (out == nullptr) return KVD_ERR_ARG;
  *out = nullptr;
  const int v = validate_config(cfg);
  if (v != KVD_OK) return v;
  kvd_ctx* c = static_cast<kvd_ctx*>(calloc(1, sizeof(kvd_ctx)));
  if (c == nullptr) return KVD_ERR_HIP;
  c->cfg = *cfg;
  c->cfg.capacity = nullptr;
  c->L = cfg->n_layers; c->B = cfg->batch; c->Hq = cfg->n_q_heads; c->Hkv = cfg->n_kv_heads;
  c->G = c->Hq / c->Hkv; c->D = cfg->head_dim; c->P = cfg->page_size; c->NP = cfg->max_pages;
  c->k = cfg->topk_pages; c->Cmax = cfg->capacity_max; c->Nc = cfg->index_centroids;
  c->Lp = cfg->physical_layers ? cfg->physical_layers : c->L;
  c->U = c->B * c->Hkv;
  c->MB = cfg->micro_batches < 1 ? 1 : cfg->micro_batches;
  if (c->MB > c->B) c->MB = c->B;
  c->bf16 = cfg->kv_dtype == KVD_BF16;
  c->tiled = kvd::slot_layout_of(c->P);
  c->wait_limit_ticks = 200000000LL;                // 2 s
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    c->n_cus = cus;
  }
  { const char* e_ = getenv("KVD_FUSE_MERGE"); c->fuse_merge = e_ ? atoi(e_) : 1; }
  { const char* e_ = getenv("KVD_SCORE_BLOCKS"); c->score_blocks = e_ ? atoi(e_) : 2048; if (c->score_blocks < 1) c->score_blocks = 1; }
  { const char* e_ = getenv("KVD_GENERIC_SELECT"); c->generic_select = e_ ? atoi(e_) : 0; }
  c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)c->D);
  c->page_bytes = (size_t)2 * c->P * c->D * 2;
  int S = cfg->attn_splits;
  // 16-token tiles of a unit's selection (pages of 4 or 8 tokens share tiles)
  const int sel_tiles = c->tiled == kvd::kLayoutPacked ? (c->k * c->P + 15) / 16 : c->k * ((c->P + 15) / 16);
  if (S == 0) {
    const int tiles = sel_tiles;
    if (c->tiled) {
      // the MFMA kernel runs one 512-thread workgroup per CU: about one workgroup per CU in the
      // grid, every wave keeping at least two tiles of 16 tokens
      S = (c->n_cus + c->U / 2) / c->U;
      if (S > tiles / 16) S = tiles / 16;
    } else {
      // the VALU kernel: one round of resident 256-thread workgroups, 8 tiles each at least
      S = (512 + c->U / 2) / c->U;
      if (S > (tiles + 7) / 8) S = (tiles + 7) / 8;
    }
    if (S > KVD_MAX_SPLITS) S = KVD_MAX_SPLITS;
    if (S < 1) S = 1;
  }
  if (S > c->k) S = c->k;
  c->S = S;
  // The one-launch step runs one workgroup per CU: 512 threads with 256 registers per lane (three
  // tile buffers in the attention role), or, for units of more than 8192 pages, 1024 threads with
  // 128.  Its attention splits: about one workgroup per CU in the first form (at least two tiles
  // per wave), four tiles per wave in the second.
  c->S1 = S;
  c->step_threads = c->NP > 8192 ? 1024 : 512;
  if (cfg->attn_splits == 0) {
    const int tiles = sel_tiles;
    int S2 = c->step_threads == 1024 ? tiles / 64 : (c->n_cus + c->U / 2) / c->U;
    const int cap = c->step_threads == 1024 ? KVD_MAX_SPLITS : tiles / 16;
    if (S2 > cap) S2 = cap;
    if (S2 > KVD_MAX_SPLITS) S2 = KVD_MAX_SPLITS;
    if (S2 < (c->k + 511) / 512) S2 = (c->k + 511) / 512;   // a split's entries are staged in LDS, 512 at most
    if (S2 > c->k) S2 = c->k;
    c->S1 = S2 < 1 ? 1 : S2;
  }
  // (room in the partials for the splits a calibration of the launch shape may try: twice the rule's)
  c->S1_max = cfg->attn_splits == 0 ? 2 * c->S1 : c->S1;
  if (c->S1_max > KVD_MAX_SPLITS) c->S1_max = KVD_MAX_SPLITS;
  if (c->S1_max > c->k) c->S1_max = c->k;
  if (c->S1_max < c->S1) c->S1_max = c->S1;
  const int Smax = c->S > c->S1_max ? c->S : c->S1_max;

  const size_t LU = (size_t)c->L * c->U;
  c->h_capacity = static_cast<int32_t*>(malloc(LU * sizeof(int32_t)));
  c->h_seq_len = static_cast<int32_t*>(malloc((size_t)c->B * sizeof(int32_t)));
  if (!c->h_capacity || !c->h_seq_len) { free_ctx(c); return KVD_ERR_HIP; }
  for (size_t i = 0; i < LU; ++i) c->h_capacity[i] = cfg->capacity ? cfg->capacity[i] : c->Cmax;
  for (int b = 0; b < c->B; ++b) c->h_seq_len[b] = c->NP * c->P;

  hipError_t e = hipSuccess;
  auto ok = [&](hipError_t r) { if (e == hipSuccess && r != hipSuccess) e = r; return e == hipSuccess; };
  const size_t Uk = (size_t)c->U * c->k;
  ok(dev_alloc(&c->d_capacity, LU)) && ok(dev_alloc(&c->d_seq_len, (size_t)c->B)) &&
      // (the page -> slot table in device memory serves the size-agnostic kernels only: the
      // register-resident path rebuilds the map in LDS from the slot array at every launch)
      (kvd_fast_path_ok(c) || ok(dev_alloc(&c->d_page_to_slot, LU * c->NP))) && ok(dev_alloc(&c->d_slot_page, LU * c->Cmax)) &&
      ok(dev_alloc(&c->d_slot_stamp, LU * c->Cmax)) && ok(dev_alloc(&c->d_resident, LU)) &&
      ok(dev_alloc(&c->d_scores, (size_t)c->U * c->NP)) && ok(dev_alloc(&c->d_sel_pages, Uk)) &&
      ok(dev_alloc(&c->d_sel_slots, Uk)) && ok(dev_alloc(&c->d_hit_mask, Uk)) && ok(dev_alloc(&c->d_evicted, Uk)) &&
      ok(dev_alloc(&c->d_counts, (size_t)c->U * 3)) && ok(dev_alloc(&c->d_miss_list, Uk * 2)) &&
      ok(dev_alloc(&c->d_miss_count, (size_t)c->U)) &&
      ok(dev_alloc(&c->d_part_acc, (size_t)c->U * Smax * c->G * c->D)) &&
      ok(dev_alloc(&c->d_part_ml, (size_t)c->U * Smax * c->G * 2)) && ok(dev_alloc(&c->d_stats, 4)) &&
      ok(dev_alloc(&c->d_attn_ticket, (size_t)c->U)) && ok(dev_alloc(&c->d_score_done, (size_t)c->U * 32)) &&
      ok(dev_alloc(&c->d_sel_entry, Uk)) && ok(dev_alloc(&c->d_timeline, (size_t)KVD_TIMELINE_MAX * 5)) &&
      ok(hipHostMalloc(reinterpret_cast<void**>(&c->error_host), sizeof(int32_t), hipHostMallocMapped)) &&
      ok(hipHostGetDevicePointer(reinterpret_cast<void**>(&c->error_dev), c->error_host, 0)) &&
      ok(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
  c->n_sets = 1;
  if (e == hipSuccess && c->L >= 2) {
    // layers in flight (kvd_step_layers): further sets of the per-step scratch
    const int want = c->L < KVD_MAX_SETS ? c->L : KVD_MAX_SETS;
    for (int i = 1; i < want && e == hipSuccess; ++i) {
      kvd_scratch& x = c->sets[i];
      c->n_sets = i + 1;                               // (what was allocated of it is freed with the context)
      ok(dev_alloc(&x.scores, (size_t)c->U * c->NP)) && ok(dev_alloc(&x.sel_pages, Uk)) && ok(dev_alloc(&x.sel_slots, Uk)) &&
          ok(dev_alloc(&x.hit_mask, Uk)) && ok(dev_alloc(&x.evicted, Uk)) && ok(dev_alloc(&x.counts, (size_t)c->U * 3)) &&
          ok(dev_alloc(&x.miss_list, Uk * 2)) && ok(dev_alloc(&x.miss_count, (size_t)c->U)) &&
          ok(dev_alloc(&x.part_acc, (size_t)c->U * Smax * c->G * c->D)) && ok(dev_alloc(&x.part_ml, (size_t)c->U * Smax * c->G * 2)) &&
          ok(dev_alloc(&x.attn_ticket, (size_t)c->U)) && ok(dev_alloc(&x.score_done, (size_t)c->U * 32)) &&
          ok(dev_alloc(&x.sel_entry, Uk)) &&
          ok(hipMemset(x.miss_count, 0, (size_t)c->U * sizeof(int32_t))) &&
          ok(hipMemset(x.attn_ticket, 0, (size_t)c->U * sizeof(int32_t))) &&
          ok(hipMemset(x.score_done, 0, (size_t)c->U * 32 * sizeof(int32_t))) &&
          ok(hipMemset(x.sel_entry, 0, Uk * sizeof(unsigned long long)));
    }
  }
  if (e == hipSuccess) ok(ensure_group_resources(c, c->n_sets > c->MB ? c->n_sets : c->MB));
  for (int i = 0; i < 12 && e == hipSuccess; ++i) ok(hipEventCreate(&c->ev_prof[i]));
  if (e == hipSuccess) ok(hipMemcpy(c->d_capacity, c->h_capacity, LU * sizeof(int32_t), hipMemcpyHostToDevice));
  if (e == hipSuccess) ok(hipMemcpy(c->d_seq_len, c->h_seq_len, (size_t)c->B * sizeof(int32_t), hipMemcpyHostToDevice));
  if (e == hipSuccess) ok(hipMemset(c->d_stats, 0, 4 * sizeof(unsigned long long)));
  if (e == hipSuccess) ok(hipMemset(c->d_miss_count, 0, (size_t)c->U * sizeof(int32_t)));
  if (e == hipSuccess) ok(hipMemset(c->d_attn_ticket, 0, (size_t)c->U * sizeof(int32_t)));
  if (e == hipSuccess) ok(hipMemset(c->d_score_done, 0, (size_t)c->U * 32 * sizeof(int32_t)));
  if (e == hipSuccess) ok(hipMemset(c->d_sel_entry, 0, Uk * sizeof(unsigned long long)));
  if (e == hipSuccess) *c->error_host = 0;
  if (e == hipSuccess) c->single_launch = kvd_wants_single_launch(c);
  if (e == hipSuccess && c->Nc > 0) ok(kvd_prepare_cluster_select());
  if (e == hipSuccess && c->Nc > 0) {
    // no page belongs to a cluster until an index is built or announced (kvd_refresh_clusters)
    ok(dev_alloc(&c->d_page_cluster, LU * c->NP));
    if (e == hipSuccess) ok(hipMemset(c->d_page_cluster, 0xff, LU * c->NP * sizeof(int32_t)));
  }
  if (e != hipSuccess) { free_ctx(c); return KVD_ERR_HIP; }
  const int r = reset_directory(c, -1);
  if (r != KVD_OK) { free_ctx(c); return r; }
  *out = c;
  return KVD_OK;
}

int kvd_destroy(kvd_ctx* ctx) {
  if (ctx == nullptr) return KVD_ERR_ARG;
  (void)hipDeviceSynchronize();
  free_ctx(ctx);
  return KVD_OK;
}

int kvd_bind_summaries(kvd_ctx* ctx, void* dev_summaries) {
  if (!ctx || !dev_summaries || !aligned16(dev_summaries)) return KVD_ERR_ARG;
  ctx->summaries = dev_summaries;
  return KVD_OK;
}

int kvd_bind_centroids(kvd_ctx* ctx, void* dev_centroids, int32_t* dev_cluster_start, int32_t* dev_cluster_pages) {
  if (!ctx || !dev_centroids || !dev_cluster_start || !dev_cluster_pages || !aligned16(dev_centroids)) return KVD_ERR_ARG;
  if (ctx->Nc == 0) return KVD_ERR_STATE;
  ctx->centroids = dev_centroids;
  ctx->cluster_start = dev_cluster_start;
  ctx->cluster_pages = dev_cluster_pages;
  return KVD_OK;
}

int kvd_build_centroids(kvd_ctx* ctx, int32_t layer, int32_t iterations, int32_t* dev_assign_trace, void* stream) {
  if (!ctx || layer < 0 || layer >= ctx->L || iterations < 1 || iterations > 64) return KVD_ERR_ARG;
  if (ctx->Nc == 0 || !ctx->summaries || !ctx->centroids) return KVD_ERR_STATE;
  HIP_TRY(ctx, kvd_run_build_centroids(ctx, layer, iterations, dev_assign_trace, static_cast<hipStream_t>(stream)));
  return KVD_OK;
}

int kvd_layout_from_clusters(kvd_ctx* ctx, int32_t layer, int32_t* host_position) {
  if (!ctx || !host_position || layer < 0 || layer >= ctx->L) return KVD_ERR_ARG;
  if (ctx->Nc == 0 || !ctx->cluster_pages) return KVD_ERR_STATE;
  const size_t n = (size_t)ctx->U * ctx->NP;
  std::vector<int32_t> listed(n);
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(listed.data(), ctx->cluster_pages + (size_t)layer * n, n * sizeof(int32_t), hipMemcpyDeviceToHost));
  for (int u = 0; u < ctx->U; ++u) {
    const int32_t* lst = listed.data() + (size_t)u * ctx->NP;
    int32_t* pos = host_position + (size_t)u * ctx->NP;
    std::fill(pos, pos + ctx->NP, -1);
    int place = 0;
    for (int i = 0; i < ctx->NP; ++i) {                      // the clusters' pages, cluster by cluster
      const int32_t p = lst[i];
      if (p < 0) continue;
      if (p >= ctx->NP || pos[p] >= 0) return KVD_ERR_STATE;
      pos[p] = place++;
    }
    for (int p = 0; p < ctx->NP; ++p)                        // pages of no cluster
      if (pos[p] < 0) pos[p] = place++;
  }
  return KVD_OK;
}

int kvd_bind_tier(kvd_ctx* ctx, kvd_tier* tier) {
  if (!ctx) return KVD_ERR_ARG;
  if (!tier) { ctx->tier = nullptr; ctx->tier_pool_dev = nullptr; return KVD_OK; }
  const kvd_tier_config* tc = kvd_tier_config_of(tier);
  if (tc->n_units != ctx->U || tc->max_pages != ctx->NP || tc->page_bytes != (int64_t)ctx->page_bytes ||
      tc->n_layers != ctx->Lp)
    return KVD_ERR_SHAPE;
  void* dptr = nullptr;
  hipError_t e = hipHostGetDevicePointer(&dptr, kvd_tier_pool_of(tier), 0);
  if (e != hipSuccess || dptr == nullptr) {
    (void)hipGetLastError();
    ctx->last_hip = (int)e;
    return KVD_ERR_ARG;
  }
  const size_t uk = (size_t)ctx->U * ctx->k;
  // (each hand-over buffer on its own: a bind that failed half way is completed by the next one)
  if (!ctx->h_miss_list)
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_miss_list), uk * 2 * sizeof(int32_t), hipHostMallocDefault));
  if (!ctx->h_miss_count)
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_miss_count), (size_t)ctx->U * sizeof(int32_t), hipHostMallocDefault));
  if (!ctx->h_src_offset)
    HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_src_offset), uk * sizeof(int64_t), hipHostMallocDefault));
  if (!ctx->d_src_offset) HIP_TRY(ctx, dev_alloc(&ctx->d_src_offset, uk));
  ctx->tier = tier;
  ctx->tier_pool_dev = static_cast<const char*>(dptr);
  return KVD_OK;
}

int kvd_refresh_clusters(kvd_ctx* ctx, int32_t layer, void* stream) {
  if (!ctx || layer < 0 || layer >= ctx->L) return KVD_ERR_ARG;
  if (ctx->Nc == 0 || !ctx->cluster_start || !ctx->cluster_pages) return KVD_ERR_STATE;
  HIP_TRY(ctx, kvd_launch_cluster_inverse(ctx, layer, static_cast<hipStream_t>(stream)));
  return KVD_OK;
}

int kvd_bind_host_store(kvd_ctx* ctx, const void* pinned_store) {
  if (!ctx || !pinned_store || !aligned16(pinned_store)) return KVD_ERR_ARG;
  void* dptr = nullptr;
  hipError_t e = hipHostGetDevicePointer(&dptr, const_cast<void*>(pinned_store), 0);
  if (e != hipSuccess || dptr == nullptr) {
    (void)hipGetLastError();
    ctx->last_hip = (int)e;
    return KVD_ERR_ARG;
  }
  ctx->store_dev = static_cast<const char*>(dptr);
  ctx->store_host = static_cast<const char*>(pinned_store);
  return KVD_OK;
}

int kvd_bind_slot_pool(kvd_ctx* ctx, void* dev_pool) {
  if (!ctx || !dev_pool || !aligned16(dev_pool)) return KVD_ERR_ARG;
  ctx->pool = static_cast<char*>(dev_pool);
  return KVD_OK;
}

int kvd_set_seq_lens(kvd_ctx* ctx, const int32_t* host_seq_len) {
  if (!ctx || !host_seq_len) return KVD_ERR_ARG;
  for (int b = 0; b < ctx->B; ++b)
    if (host_seq_len[b] < 1 || (long long)host_seq_len[b] > (long long)ctx->NP * ctx->P) return KVD_ERR_SHAPE;
  memcpy(ctx->h_seq_len, host_seq_len, (size_t)ctx->B * sizeof(int32_t));
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(ctx->d_seq_len, ctx->h_seq_len, (size_t)ctx->B * sizeof(int32_t), hipMemcpyHostToDevice));
  return KVD_OK;
}

int kvd_build_summaries(kvd_ctx* ctx, int32_t layer, void* stream) {
  if (!ctx || layer < 0 || layer >= ctx->L) return KVD_ERR_ARG;
  if (!ctx->summaries || !ctx->store_dev) return KVD_ERR_STATE;
  HIP_TRY(ctx, kvd_launch_build_summaries(ctx, layer, static_cast<hipStream_t>(stream)));
  return KVD_OK;
}

int kvd_append_kv(kvd_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, void* stream) {
  if (!ctx || !k_new || !v_new || layer < 0 || layer >= ctx->L || !aligned16(k_new) || !aligned16(v_new)) return KVD_ERR_ARG;
  if (!ctx->summaries || !ctx->pool || !ctx->store_dev) return KVD_ERR_STATE;
  if (ctx->Lp != ctx->L) return KVD_ERR_STATE;       // layers that share a stored layer cannot each append to it
  for (int b = 0; b < ctx->B; ++b)
    if ((long long)ctx->h_seq_len[b] >= (long long)ctx->NP * ctx->P) return KVD_ERR_SHAPE;
  HIP_TRY(ctx, kvd_launch_append(ctx, layer, k_new, v_new, static_cast<hipStream_t>(stream)));
  if (ctx->tier != nullptr) {
    // the backing file (and the pool's copy) must hold the token too: carry its K row and V row over
    // from the host store, which the kernel has just written
    HIP_TRY(ctx, hipStreamSynchronize(static_cast<hipStream_t>(stream)));
    const size_t row = (size_t)ctx->D * 2;
    for (int u = 0; u < ctx->U; ++u) {
      const int t = ctx->h_seq_len[u / ctx->Hkv];
      const int page = t / ctx->P, r = t % ctx->P;
      const char* pg = ctx->store_host + (((size_t)layer * ctx->U + u) * ctx->NP + page) * ctx->page_bytes;
      int rc = kvd_tier_patch_page(ctx->tier, layer, u, page, (int64_t)r * row, pg + (size_t)r * row, (int64_t)row);
      if (rc == KVD_OK)
        rc = kvd_tier_patch_page(ctx->tier, layer, u, page, (int64_t)(ctx->P + r) * row, pg + (size_t)(ctx->P + r) * row,
                                 (int64_t)row);
      if (rc != KVD_OK) return rc;
    }
  }
  return KVD_OK;
}

int kvd_advance(kvd_ctx* ctx, void* stream) {
  if (!ctx) return KVD_ERR_ARG;
  for (int b = 0; b < ctx->B; ++b)
    if ((long long)ctx->h_seq_len[b] >= (long long)ctx->NP * ctx->P) return KVD_ERR_SHAPE;
  HIP_TRY(ctx, kvd_launch_advance(ctx, static_cast<hipStream_t>(stream)));
  for (int b = 0; b < ctx->B; ++b) ++ctx->h_seq_len[b];
  return KVD_OK;
}

int kvd_cache_reset(kvd_ctx* ctx) {
  if (!ctx) return KVD_ERR_ARG;
  HIP_TRY(ctx, hipDeviceSynchronize());
  const int r = clear_step_flags(ctx);
  if (r != KVD_OK) return r;
  *ctx->error_host = 0;
  return reset_directory(ctx, -1);
}

// Checks a [U][Cmax] slot_page image and derives page_to_slot / resident from it.
static int install_directory(kvd_ctx* c, int layer, const std::vector<int32_t>& slot_page,
                             const std::vector<int32_t>& slot_stamp) {
  const size_t U = c->U, NP = c->NP, Cmax = c->Cmax;
  std::vector<int32_t> p2s(U * NP, -1), resident(U, 0);
  for (size_t u = 0; u < U; ++u) {
    const int cap = c->h_capacity[(size_t)layer * U + u];
    for (size_t s = 0; s < Cmax; ++s) {
      const int32_t p = slot_page[u * Cmax + s];
      if (p < 0) continue;
      if ((int)s >= cap || (size_t)p >= NP || p2s[u * NP + p] >= 0) return KVD_ERR_STATE;
      p2s[u * NP + p] = (int32_t)s;
      ++resident[u];
    }
  }
  const size_t lu = (size_t)layer * U;
  HIP_TRY(c, hipDeviceSynchronize());
  if (c->d_page_to_slot)
    HIP_TRY(c, hipMemcpy(c->d_page_to_slot + lu * NP, p2s.data(), U * NP * sizeof(int32_t), hipMemcpyHostToDevice));
  HIP_TRY(c, hipMemcpy(c->d_slot_page + lu * Cmax, slot_page.data(), U * Cmax * sizeof(int32_t), hipMemcpyHostToDevice));
  HIP_TRY(c, hipMemcpy(c->d_slot_stamp + lu * Cmax, slot_stamp.data(), U * Cmax * sizeof(int32_t), hipMemcpyHostToDevice));
  HIP_TRY(c, hipMemcpy(c->d_resident + lu, resident.data(), U * sizeof(int32_t), hipMemcpyHostToDevice));
  HIP_TRY(c, kvd_launch_refill(c, layer, nullptr));
  HIP_TRY(c, hipDeviceSynchronize());
  return KVD_OK;
}

int kvd_cache_warm(kvd_ctx* ctx, int32_t layer, const int32_t* host_pages, const int32_t* host_counts) {
  if (!ctx || !host_pages || !host_counts || layer < 0 || layer >= ctx->L) return KVD_ERR_ARG;
  if (!ctx->pool || !ctx->store_dev) return KVD_ERR_STATE;
  const size_t U = ctx->U, Cmax = ctx->Cmax;
  std::vector<int32_t> slot_page(U * Cmax, -1), slot_stamp(U * Cmax, -1);
  size_t off = 0;
  for (size_t u = 0; u < U; ++u) {
    const int n = host_counts[u];
    if (n < 0) return KVD_ERR_ARG;
    if (n > ctx->h_capacity[(size_t)layer * U + u]) return KVD_ERR_CAPACITY;
    for (int i = 0; i < n; ++i) {
      const int32_t p = host_pages[off + i];
      if (p < 0 || p >= ctx->NP) return KVD_ERR_ARG;
      slot_page[u * Cmax + i] = p;
    }
    off += (size_t)n;
  }
  const int r = install_directory(ctx, layer, slot_page, slot_stamp);
  return r == KVD_ERR_STATE ? KVD_ERR_ARG : r;       // a repeated page in a warm list is a bad argument
}

int kvd_cache_export(kvd_ctx* ctx, int32_t layer, int32_t* host_slot_page, int32_t* host_slot_stamp) {
  if (!ctx || !host_slot_page || !host_slot_stamp || layer < 0 || layer >= ctx->L) return KVD_ERR_ARG;
  const size_t n = (size_t)ctx->U * ctx->Cmax, lu = (size_t)layer * ctx->U;
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(host_slot_page, ctx->d_slot_page + lu * ctx->Cmax, n * sizeof(int32_t), hipMemcpyDeviceToHost));
  HIP_TRY(ctx, hipMemcpy(host_slot_stamp, ctx->d_slot_stamp + lu * ctx->Cmax, n * sizeof(int32_t), hipMemcpyDeviceToHost));
  return KVD_OK;
}

int kvd_cache_import(kvd_ctx* ctx, int32_t layer, const int32_t* host_slot_page, const int32_t* host_slot_stamp) {
  if (!ctx || !host_slot_page || !host_slot_stamp || layer < 0 || layer >= ctx->L) return KVD_ERR_ARG;
  if (!ctx->pool || !ctx->store_dev) return KVD_ERR_STATE;
  const size_t n = (size_t)ctx->U * ctx->Cmax;
  std::vector<int32_t> slot_page(host_slot_page, host_slot_page + n), slot_stamp(host_slot_stamp, host_slot_stamp + n);
  return install_directory(ctx, layer, slot_page, slot_stamp);
}

int kvd_score_select(kvd_ctx* ctx, int32_t layer, const void* q, int32_t* sel_pages, float* scores, void* stream) {
  if (!ctx || !q || !sel_pages || layer < 0 || layer >= ctx->L || !aligned16(q)) return KVD_ERR_ARG;
  if (ctx->Nc > 0 ? !ctx->centroids : !ctx->summaries) return KVD_ERR_STATE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* sc = scores ? scores : ctx->d_scores;
  ctx->last_scores = sc;
  HIP_TRY(ctx, kvd_launch_score(ctx, layer, q, sc, 0, ctx->U, s));
  if (ctx->Nc > 0)
    HIP_TRY(ctx, kvd_launch_cluster_select(ctx, layer, sc, sel_pages, 0, ctx->U, s));
  else if (kvd_fast_path_ok(ctx))
    HIP_TRY(ctx, kvd_launch_select_resolve(ctx, layer, 0, true, false, false, sc, sel_pages, nullptr, nullptr, nullptr,
                                           nullptr, 0, ctx->U, s));
  else
    HIP_TRY(ctx, kvd_launch_select(ctx, sc, sel_pages, 0, ctx->U, s));
  return KVD_OK;
}

int kvd_cache_resolve(kvd_ctx* ctx, int32_t layer, int32_t step, const int32_t* sel_pages, int32_t* sel_slots,
                      int32_t* hit_mask, int32_t* evicted, int32_t* counts, int32_t do_gather, void* stream) {
  if (!ctx || !sel_pages || !sel_slots || layer < 0 || layer >= ctx->L) return KVD_ERR_ARG;
  if (do_gather && (!ctx->pool || !ctx->store_dev)) return KVD_ERR_STATE;
  if (ctx->cfg.policy == KVD_EVICT_LOOKAHEAD && ctx->last_scores == nullptr) return KVD_ERR_STATE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* hm = hit_mask ? hit_mask : ctx->d_hit_mask;
  int32_t* ev = evicted ? evicted : ctx->d_evicted;
  int32_t* cn = counts ? counts : ctx->d_counts;
  if (kvd_fast_path_ok(ctx)) {
    HIP_TRY(ctx, kvd_launch_select_resolve(ctx, layer, step, false, true, do_gather != 0, ctx->last_scores,
                                           const_cast<int32_t*>(sel_pages), sel_slots, hm, ev, cn, 0, ctx->U, s));
  } else {
    HIP_TRY(ctx, kvd_launch_resolve(ctx, layer, step, sel_pages, sel_slots, hm, ev, cn, 0, ctx->U, s));
    if (do_gather) HIP_TRY(ctx, kvd_launch_gather(ctx, layer, 0, ctx->U, s));
  }
  ++ctx->n_steps;
  return KVD_OK;
}

int kvd_sparse_decode_attn(kvd_ctx* ctx, int32_t layer, const void* q, const int32_t* sel_pages,
                           const int32_t* sel_slots, float* out, float* lse, void* stream) {
  if (!ctx || !q || !sel_pages || !sel_slots || !out || layer < 0 || layer >= ctx->L || !aligned16(q))
    return KVD_ERR_ARG;
  if (!ctx->pool) return KVD_ERR_STATE;
  HIP_TRY(ctx, kvd_launch_attend(ctx, layer, q, sel_pages, sel_slots, out, lse, 0, ctx->U, static_cast<hipStream_t>(stream)));
  return KVD_OK;
}

// Selection + directory update + fetch for units [u0, u1): one fused kernel when the sizes allow
// the register-resident path, else the three size-agnostic kernels.
static hipError_t launch_select_resolve_fetch(kvd_ctx* c, int layer, int step, int u0, int u1, hipStream_t s,
                                              bool fetch = true) {
  if (c->Nc > 0) {
    // hierarchical index: clusters -> pages, then the directory update and the fetch
    hipError_t e = kvd_launch_cluster_select(c, layer, c->d_scores, c->d_sel_pages, u0, u1, s);
    if (e != hipSuccess) return e;
    if (kvd_fast_path_ok(c))
      return kvd_launch_select_resolve(c, layer, step, false, true, fetch, c->d_scores, c->d_sel_pages, c->d_sel_slots,
                                       c->d_hit_mask, c->d_evicted, c->d_counts, u0, u1, s);
    e = kvd_launch_resolve(c, layer, step, c->d_sel_pages, c->d_sel_slots, c->d_hit_mask, c->d_evicted, c->d_counts, u0,
                           u1, s);
    if (e != hipSuccess || !fetch) return e;
    return kvd_launch_gather(c, layer, u0, u1, s);
  }
  if (kvd_fast_path_ok(c))
    return kvd_launch_select_resolve(c, layer, step, true, true, fetch, c->d_scores, c->d_sel_pages, c->d_sel_slots,
                                     c->d_hit_mask, c->d_evicted, c->d_counts, u0, u1, s);
  hipError_t e = kvd_launch_select(c, c->d_scores, c->d_sel_pages, u0, u1, s);
  if (e != hipSuccess) return e;
  e = kvd_launch_resolve(c, layer, step, c->d_sel_pages, c->d_sel_slots, c->d_hit_mask, c->d_evicted, c->d_counts, u0,
                         u1, s);
  if (e != hipSuccess || !fetch) return e;
  return kvd_launch_gather(c, layer, u0, u1, s);
}

// One layer-step with every stage bracketed by HIP events on the caller's stream; waits for the
// step and accumulates the per-stage times.  Stages run for the whole batch, one after another.
static int step_profiled(kvd_ctx* c, int layer, int step, const void* q, float* out, float* lse, hipStream_t s) {
  hipEvent_t* ev = c->ev_prof;
  const bool fused = kvd_fast_path_ok(c) || c->Nc > 0;
  HIP_TRY(c, hipEventRecord(ev[0], s));
  HIP_TRY(c, kvd_launch_score(c, layer, q, c->d_scores, 0, c->U, s));
  HIP_TRY(c, hipEventRecord(ev[1], s));
  if (fused) {
    HIP_TRY(c, launch_select_resolve_fetch(c, layer, step, 0, c->U, s));
    HIP_TRY(c, hipEventRecord(ev[2], s));
    HIP_TRY(c, hipEventRecord(ev[3], s));
  } else {
    HIP_TRY(c, kvd_launch_select(c, c->d_scores, c->d_sel_pages, 0, c->U, s));
    HIP_TRY(c, kvd_launch_resolve(c, layer, step, c->d_sel_pages, c->d_sel_slots, c->d_hit_mask, c->d_evicted,
                                  c->d_counts, 0, c->U, s));
    HIP_TRY(c, hipEventRecord(ev[2], s));
    HIP_TRY(c, kvd_launch_gather(c, layer, 0, c->U, s));
    HIP_TRY(c, hipEventRecord(ev[3], s));
  }
  const bool own_merge = c->fuse_merge || c->S == 1;   // the attention kernel merges its own splits
  HIP_TRY(c, kvd_launch_attend(c, layer, q, c->d_sel_pages, c->d_sel_slots, out, lse, 0, c->U, s, own_merge ? nullptr : ev[4]));
  HIP_TRY(c, hipEventRecord(ev[5], s));
  HIP_TRY(c, hipEventSynchronize(ev[5]));
  float ms = 0.f;
  HIP_TRY(c, hipEventElapsedTime(&ms, ev[0], ev[1])); c->ms_score += ms;
  HIP_TRY(c, hipEventElapsedTime(&ms, ev[1], ev[2])); c->ms_select_resolve += ms;
  HIP_TRY(c, hipEventElapsedTime(&ms, ev[2], ev[3])); c->ms_gather += ms;
  if (own_merge) {
    HIP_TRY(c, hipEventElapsedTime(&ms, ev[3], ev[5])); c->ms_attend += ms;
  } else {
    HIP_TRY(c, hipEventElapsedTime(&ms, ev[3], ev[4])); c->ms_attend += ms;
    HIP_TRY(c, hipEventElapsedTime(&ms, ev[4], ev[5])); c->ms_merge += ms;
  }
  HIP_TRY(c, hipEventElapsedTime(&ms, ev[0], ev[5])); c->ms_total += ms;
  ++c->profiled_steps;
  return KVD_OK;
}

// One layer-step in the context's current form, enqueued on s (and, with micro-batches, on the
// library's streams, forked from and joined back into s).
static int enqueue_step(kvd_ctx* c, int layer, int step, const void* q, float* out, float* lse, hipStream_t s, bool groups) {
  ++c->n_steps;
  c->last_scores = c->d_scores;
  if (c->single_launch) {
    HIP_TRY(c, kvd_launch_step(c, layer, 1, step, q, out, lse, s));
    return KVD_OK;
  }
  if (c->MB <= 1 || !groups) {
    HIP_TRY(c, kvd_launch_score(c, layer, q, c->d_scores, 0, c->U, s));
    HIP_TRY(c, launch_select_resolve_fetch(c, layer, step, 0, c->U, s));
    HIP_TRY(c, kvd_launch_attend(c, layer, q, c->d_sel_pages, c->d_sel_slots, out, lse, 0, c->U, s));
    return KVD_OK;
  }
  // Micro-batches (SFC Disaggregation): group i of the sequences runs select -> fetch -> attend as
  // its own chain on pipeline stream i % (1 + KVD_PIPE_STREAMS) (stream 0 is the caller's), so the
  // latency-bound selection and the host-link fetch of one group overlap the bandwidth-bound
  // kernels of the others.  Scoring is chained group to group so that the groups start staggered.
  HIP_TRY(c, hipEventRecord(c->ev_fork, s));
  for (int i = 0; i < KVD_PIPE_STREAMS; ++i) HIP_TRY(c, hipStreamWaitEvent(c->side[i], c->ev_fork, 0));
  for (int i = 0; i < c->MB; ++i) {
    const int u0 = (int)(((long long)i * c->B) / c->MB) * c->Hkv;
    const int u1 = (int)(((long long)(i + 1) * c->B) / c->MB) * c->Hkv;
    const int lane = i % (1 + KVD_PIPE_STREAMS);
    hipStream_t st = lane == 0 ? s : c->side[lane - 1];
    if (i > 0) HIP_TRY(c, hipStreamWaitEvent(st, c->ev_score[i - 1], 0));
    HIP_TRY(c, kvd_launch_score(c, layer, q, c->d_scores, u0, u1, st));
    HIP_TRY(c, hipEventRecord(c->ev_score[i], st));
    HIP_TRY(c, launch_select_resolve_fetch(c, layer, step, u0, u1, st));
    HIP_TRY(c, kvd_launch_attend(c, layer, q, c->d_sel_pages, c->d_sel_slots, out, lse, u0, u1, st));
    if (lane != 0) HIP_TRY(c, hipEventRecord(c->ev_done[i], st));
  }
  for (int i = 0; i < c->MB; ++i)
    if (i % (1 + KVD_PIPE_STREAMS) != 0) HIP_TRY(c, hipStreamWaitEvent(s, c->ev_done[i], 0));
  return KVD_OK;
}

int kvd_step(kvd_ctx* ctx, int32_t layer, int32_t step, const void* q, float* out, float* lse, void* stream) {
  if (!ctx || !q || !out || layer < 0 || layer >= ctx->L || !aligned16(q)) return KVD_ERR_ARG;
  if (!ctx->summaries || !ctx->pool || !ctx->store_dev || (ctx->Nc > 0 && !ctx->centroids)) return KVD_ERR_STATE;
  kvd_ctx* c = ctx;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (*c->error_host != 0) return recover_from_wait_timeout(c);   // an earlier one-launch step gave up waiting
  if (c->profiling == 1) {
    ++c->n_steps;
    c->last_scores = c->d_scores;
    return step_profiled(c, layer, step, q, out, lse, s);
  }
  return enqueue_step(c, layer, step, q, out, lse, s, true);
}

int kvd_step_layers(kvd_ctx* ctx, int32_t layer0, int32_t n_layers, int32_t step, const void* q_layers, float* out_layers,
                    float* lse_layers, void* stream) {
  if (!ctx || !q_layers || !out_layers || layer0 < 0 || n_layers < 1 || (long long)layer0 + n_layers > ctx->L ||
      !aligned16(q_layers))
    return KVD_ERR_ARG;
  if (!ctx->summaries || !ctx->pool || !ctx->store_dev || (ctx->Nc > 0 && !ctx->centroids)) return KVD_ERR_STATE;
  kvd_ctx* c = ctx;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (*c->error_host != 0) return recover_from_wait_timeout(c);
  const size_t rows = (size_t)c->B * c->Hq;
  const char* q = static_cast<const char*>(q_layers);
  auto q_of = [&](int i) { return static_cast<const void*>(q + (size_t)i * rows * c->D * 2); };
  auto out_of = [&](int i) { return out_layers + (size_t)i * rows * c->D; };
  auto lse_of = [&](int i) { return lse_layers ? lse_layers + (size_t)i * rows : nullptr; };
  if (c->single_launch && c->profiling == 0 && c->n_sets >= 2 && n_layers >= 2) {
    // one launch for up to n_sets layers at a time, the layers pipelined through the compute units by
    // the launch's block order; everything on the caller's stream
    int done = 0;
    while (done < n_layers) {
      const int n = n_layers - done < c->n_sets ? n_layers - done : c->n_sets;
      c->n_steps += (uint64_t)n;
      c->last_scores = nullptr;
      if (n == 1) use_scratch_set(c, 0);
      HIP_TRY(c, kvd_launch_step(c, layer0 + done, n, step, q_of(done), out_of(done), lse_of(done), s));
      use_scratch_set(c, n - 1);                       // kvd_step_trace reports the last layer
      c->last_scores = c->d_scores;
      done += n;
    }
    return KVD_OK;
  }
  int lanes = c->n_sets < n_layers ? c->n_sets : n_layers;
  if (lanes > KVD_LAYER_LANES) lanes = KVD_LAYER_LANES;
  if (lanes < 2 || c->profiling != 0) {
    for (int i = 0; i < n_layers; ++i) {
      const int r = kvd_step(c, layer0 + i, step, q_of(i), out_of(i), lse_of(i), stream);
      if (r != KVD_OK) return r;
    }
    return KVD_OK;
  }
  // Layer i runs in lane i % lanes: lane 0 is the caller's stream, the others are the library's,
  // each with its own set of per-step scratch, so that the fetch of one layer's missed pages
  // overlaps the kernels of the next ones.  Layers `lanes` apart follow each other on one stream,
  // so a scratch set is never in use twice.
  HIP_TRY(c, hipEventRecord(c->ev_fork, s));
  for (int j = 1; j < lanes; ++j) HIP_TRY(c, hipStreamWaitEvent(c->side[j - 1], c->ev_fork, 0));
  int r = KVD_OK;
  for (int i = 0; i < n_layers && r == KVD_OK; ++i) {
    const int lane = i % lanes;
    use_scratch_set(c, lane);
    r = enqueue_step(c, layer0 + i, step, q_of(i), out_of(i), lse_of(i), lane == 0 ? s : c->side[lane - 1], false);
  }
  // (the context keeps the scratch set of the last layer enqueued: kvd_step_trace reports that layer)
  hipError_t e = hipSuccess;
  for (int j = 1; j < lanes; ++j) {
    if (e == hipSuccess) e = hipEventRecord(c->ev_done[j], c->side[j - 1]);
    if (e == hipSuccess) e = hipStreamWaitEvent(s, c->ev_done[j], 0);
  }
  if (r != KVD_OK) return r;
  HIP_TRY(c, e);
  return KVD_OK;
}

int kvd_step_tiered(kvd_ctx* ctx, int32_t layer, int32_t step, const void* q, float* out, float* lse, void* stream) {
  if (!ctx || !q || !out || layer < 0 || layer >= ctx->L || !aligned16(q)) return KVD_ERR_ARG;
  if (!ctx->summaries || !ctx->pool || !ctx->tier || (ctx->Nc > 0 && !ctx->centroids)) return KVD_ERR_STATE;
  kvd_ctx* c = ctx;
  hipStream_t s = static_cast<hipStream_t>(stream);
  ++c->n_steps;
  c->last_scores = c->d_scores;
  // (1) select, and the directory update, on the GPU; nothing is fetched yet
  HIP_TRY(c, kvd_launch_score(c, layer, q, c->d_scores, 0, c->U, s));
  HIP_TRY(c, launch_select_resolve_fetch(c, layer, step, 0, c->U, s, false));
  // (2) the misses go to the host, which reads the extents that hold them into its pool
  const size_t uk = (size_t)c->U * c->k;
  HIP_TRY(c, hipMemcpyAsync(c->h_miss_count, c->d_miss_count, (size_t)c->U * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipMemcpyAsync(c->h_miss_list, c->d_miss_list, uk * 2 * sizeof(int32_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  const int rc = kvd_tier_fetch(c->tier, layer % c->Lp, step, c->h_miss_list, c->h_miss_count, c->k, c->h_src_offset);
  if (rc != KVD_OK) {
    // the directory already names slots for pages that will not arrive: empty the layer's window
    const int rr = reset_directory(c, layer);
    return rr != KVD_OK ? rr : rc;
  }
  // (3) pool -> slots, then attention
  HIP_TRY(c, hipMemcpyAsync(c->d_src_offset, c->h_src_offset, uk * sizeof(int64_t), hipMemcpyHostToDevice, s));
  HIP_TRY(c, kvd_launch_gather(c, layer, 0, c->U, s, c->tier_pool_dev, c->d_src_offset));
  HIP_TRY(c, kvd_launch_attend(c, layer, q, c->d_sel_pages, c->d_sel_slots, out, lse, 0, c->U, s));
  return KVD_OK;
}

int kvd_step_trace(kvd_ctx* ctx, int32_t* sel_pages, int32_t* sel_slots, int32_t* hit_mask, int32_t* evicted,
                   int32_t* counts, float* scores, void* stream) {
  if (!ctx) return KVD_ERR_ARG;
  if (*ctx->error_host != 0) return KVD_ERR_STATE;    // a one-launch step that has already ended gave up waiting: its trace is not one
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t uk = (size_t)ctx->U * ctx->k * sizeof(int32_t);
  if (sel_pages) HIP_TRY(ctx, hipMemcpyAsync(sel_pages, ctx->d_sel_pages, uk, hipMemcpyDeviceToDevice, s));
  if (sel_slots) HIP_TRY(ctx, hipMemcpyAsync(sel_slots, ctx->d_sel_slots, uk, hipMemcpyDeviceToDevice, s));
  if (hit_mask) HIP_TRY(ctx, hipMemcpyAsync(hit_mask, ctx->d_hit_mask, uk, hipMemcpyDeviceToDevice, s));
  if (evicted) HIP_TRY(ctx, hipMemcpyAsync(evicted, ctx->d_evicted, uk, hipMemcpyDeviceToDevice, s));
  if (counts)
    HIP_TRY(ctx, hipMemcpyAsync(counts, ctx->d_counts, (size_t)ctx->U * 3 * sizeof(int32_t), hipMemcpyDeviceToDevice, s));
  if (scores)
    HIP_TRY(ctx, hipMemcpyAsync(scores, ctx->d_scores, (size_t)ctx->U * ctx->NP * sizeof(float), hipMemcpyDeviceToDevice, s));
  return KVD_OK;
}

int kvd_set_profiling(kvd_ctx* ctx, int32_t on) {
  if (!ctx) return KVD_ERR_ARG;
  if (on < 0 || on > 2) return KVD_ERR_ARG;
  ctx->profiling = on;
  return KVD_OK;
}

int kvd_set_step_form(kvd_ctx* ctx, int32_t form) {
  if (!ctx) return KVD_ERR_ARG;
  if (form < -1 || form > KVD_MAX_MICRO) return KVD_ERR_SHAPE;
  if (form == -1 && !kvd_single_launch_ok(ctx)) return KVD_ERR_SHAPE;
  HIP_TRY(ctx, hipDeviceSynchronize());
  ctx->cfg.micro_batches = form;
  ctx->MB = form < 1 ? 1 : form;
  if (ctx->MB > ctx->B) ctx->MB = ctx->B;
  HIP_TRY(ctx, ensure_group_resources(ctx, ctx->MB));
  ctx->single_launch = kvd_wants_single_launch(ctx);
  return KVD_OK;
}

int kvd_calibrate_step_form(kvd_ctx* ctx, int32_t layer, int32_t first_step, const void* q_steps, int32_t n_queries,
                            int32_t steps_per_form, float* out, void* stream, int32_t* chosen_form,
                            float* ms_per_step_or_null) {
  if (!ctx || !q_steps || !out || !chosen_form || layer < 0 || layer >= ctx->L || n_queries < 1 || steps_per_form < 1 ||
      !aligned16(q_steps))
    return KVD_ERR_ARG;
  if (!ctx->summaries || !ctx->pool || !ctx->store_dev || ctx->profiling != 0) return KVD_ERR_STATE;   // (profiled steps all run as one chain)
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int candidates[4] = {1, 2, 4, -1};
  const size_t q_bytes = (size_t)ctx->B * ctx->Hq * ctx->D * 2;
  hipEvent_t e0 = ctx->ev_prof[10], e1 = ctx->ev_prof[11];
  bool runs[4];
  double total_ms[4] = {0.0, 0.0, 0.0, 0.0};
  for (int ci = 0; ci < 4; ++ci)
    runs[ci] = !((candidates[ci] == -1 && !kvd_single_launch_ok(ctx)) || candidates[ci] > ctx->B);
  // Every form replays the same steps from the same cache: the directory as it is now is kept on
  // the host and put back (slots refilled from the host store) before each replay, so that all
  // forms see the same misses — the time of a step follows its misses, which vary more from step
  // to step than the forms differ.  Two rounds, the forms in order and then in reverse order; a
  // form's time is the smaller of its two (what disturbs a run only ever adds time).  The first
  // step of a replay is not timed (first use of a form creates streams and loads code).
  const size_t n_dir = (size_t)ctx->U * ctx->Cmax;
  std::vector<int32_t> slot_page0(n_dir), slot_stamp0(n_dir);
  int r = kvd_cache_export(ctx, layer, slot_page0.data(), slot_stamp0.data());
  if (r != KVD_OK) return r;
  double best_of[4] = {-1.0, -1.0, -1.0, -1.0};
  bool first = true;
  for (int pass = 0; pass < 2; ++pass) {
    for (int k = 0; k < 4; ++k) {
      const int ci = pass == 0 ? k : 3 - k;
      if (!runs[ci]) continue;
      if (!first) {
        r = install_directory(ctx, layer, slot_page0, slot_stamp0);
        if (r != KVD_OK) return r;
      }
      first = false;
      r = kvd_set_step_form(ctx, candidates[ci]);
      if (r != KVD_OK) return r;
      for (int i = 0; i <= steps_per_form; ++i) {
        if (i == 1) HIP_TRY(ctx, hipEventRecord(e0, s));
        r = kvd_step(ctx, layer, first_step + i, static_cast<const char*>(q_steps) + (size_t)(i % n_queries) * q_bytes, out,
                     nullptr, s);
        if (r != KVD_OK) return r;
      }
      HIP_TRY(ctx, hipEventRecord(e1, s));
      HIP_TRY(ctx, hipEventSynchronize(e1));
      float ms = 0.f;
      HIP_TRY(ctx, hipEventElapsedTime(&ms, e0, e1));
      if (best_of[ci] < 0.0 || ms < best_of[ci]) best_of[ci] = ms;
    }
  }
  for (int ci = 0; ci < 4; ++ci) total_ms[ci] = best_of[ci];
  int best = 1;
  double best_ms = -1.0;
  for (int ci = 0; ci < 4; ++ci) {
    const double ms = runs[ci] ? total_ms[ci] / steps_per_form : -1.0;
    if (ms_per_step_or_null) ms_per_step_or_null[ci] = (float)ms;
    if (runs[ci] && (best_ms < 0.0 || ms < best_ms)) { best_ms = ms; best = candidates[ci]; }
  }
  *chosen_form = best;
  return kvd_set_step_form(ctx, best);
}

int kvd_set_step_shape(kvd_ctx* ctx, int32_t multi_layer, int32_t passes, int32_t scoring_workgroups, int32_t attn_splits,
                       int32_t groups) {
  if (!ctx) return KVD_ERR_ARG;
  if (passes < 0 || scoring_workgroups < 0 || attn_splits < 0 || groups < 0) return KVD_ERR_SHAPE;
  if (scoring_workgroups > ctx->n_cus || groups > 8) return KVD_ERR_SHAPE;   // (more groups than units: as many groups as units)
  const kvd_shape want = {passes, scoring_workgroups, attn_splits, groups};
  if (!kvd_step_shape_ok(ctx, kvd_step_shape(ctx, multi_layer, &want))) return KVD_ERR_SHAPE;
  HIP_TRY(ctx, hipDeviceSynchronize());               // (launches in flight keep the shape they were given)
  ctx->shape[multi_layer ? 1 : 0] = want;
  return KVD_OK;
}

int kvd_get_step_shape(const kvd_ctx* ctx, int32_t multi_layer, int32_t* shape) {
  if (!ctx || !shape) return KVD_ERR_ARG;
  const kvd_shape e = kvd_step_shape(ctx, multi_layer);
  shape[0] = e.passes; shape[1] = e.n_score; shape[2] = e.splits; shape[3] = e.groups;
  return KVD_OK;
}

int kvd_calibrate_step_shape(kvd_ctx* ctx, int32_t layer, int32_t n_layers, int32_t step, const void* q_layers, float* out_layers,
                             void* stream, int32_t launches_per_shape, int32_t* chosen_shape, float* us_chosen, float* us_rule) {
  if (!ctx || !q_layers || !out_layers || layer < 0 || n_layers < 1 || (long long)layer + n_layers > ctx->L ||
      launches_per_shape < 1 || !aligned16(q_layers))
    return KVD_ERR_ARG;
  if (!ctx->summaries || !ctx->pool || !ctx->store_dev || (ctx->Nc > 0 && !ctx->centroids)) return KVD_ERR_STATE;
  if (!ctx->single_launch || ctx->profiling != 0) return KVD_ERR_STATE;
  kvd_ctx* c = ctx;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0 = c->ev_prof[10], e1 = c->ev_prof[11];
  const int multi = n_layers > 1 ? 1 : 0;
  auto one = [&]() -> int {
    return multi ? kvd_step_layers(c, layer, n_layers, step, q_layers, out_layers, nullptr, s)
                 : kvd_step(c, layer, step, q_layers, out_layers, nullptr, s);
  };
  // the step once as it is: afterwards every page the queries select is resident, and the replays
  // below are pure GPU work
  int r = one();
  if (r != KVD_OK) return r;
  HIP_TRY(c, hipStreamSynchronize(s));
  // Times `n` replays in the current shape, after two untimed ones; microseconds per layer-step.
  auto time_shape = [&](int n, double* us) -> int {
    for (int i = 0; i < n + 2; ++i) {
      if (i == 2) HIP_TRY(c, hipEventRecord(e0, s));
      const int rr = one();
      if (rr != KVD_OK) return rr;
    }
    HIP_TRY(c, hipEventRecord(e1, s));
    HIP_TRY(c, hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&ms, e0, e1));
    *us = 1e3 * ms / ((double)n * n_layers);
    return KVD_OK;
  };
  struct Timed { kvd_shape shape; double us; bool is_rule; };
  std::vector<Timed> shapes;
  const kvd_shape nothing = {0, 0, 0, 0};
  const kvd_shape rule = kvd_step_shape(c, multi, &nothing);
  auto same = [](const kvd_shape& a, const kvd_shape& b) {
    return a.passes == b.passes && a.n_score == b.n_score && a.splits == b.splits && a.groups == b.groups;
  };
  auto add = [&](const kvd_shape& want) {
    const kvd_shape e = kvd_step_shape(c, multi, &want);
    if (!kvd_step_shape_ok(c, e)) return;
    for (const Timed& x : shapes)
      if (same(x.shape, e)) return;
    shapes.push_back({e, 0.0, false});
  };
  add(nothing);
  // The grid: scoring workgroups from every compute unit (no slot left to the selections while a
  // group is scored) down to a quarter of them; 1..4 passes; splits from a quarter of the rule's to
  // twice; a layer in 1, 2 or 4 groups (launches of several layers, which the layers already
  // pipeline: one group).
  const int sr = rule.splits;
  for (int g : {1, 2, 4}) {
    if (multi && g > 1) break;
    for (int sp : {sr / 4, sr / 2, (3 * sr) / 4, sr, (3 * sr) / 2, 2 * sr})
      for (int eighths = 8; eighths >= 2; --eighths)
        for (int p = 1; p <= 4; ++p)
          if (sp >= 1) add({p, c->n_cus * eighths / 8, sp, g});
  }
  auto apply = [&](const kvd_shape& x) { c->shape[multi] = x; };
  const kvd_shape before = c->shape[multi];
  for (Timed& x : shapes) {
    apply(x.shape);
    r = time_shape(launches_per_shape, &x.us);
    if (r != KVD_OK) { apply(before); return r; }
  }
  // the eight fastest and the rule's shape once more, three times as long; the smaller of a
  // shape's two times counts (what disturbs a run only ever adds time).  Another shape replaces the
  // rule's only if it is more than 1.5 % faster: differences below that are within what two timings
  // of one shape differ by, and the replayed query is not every query.
  shapes[0].is_rule = true;
  std::sort(shapes.begin(), shapes.end(), [](const Timed& a, const Timed& b) { return a.us < b.us; });
  const size_t top = shapes.size() < 8 ? shapes.size() : 8;
  size_t rule_at = 0;
  for (size_t i = 0; i < shapes.size(); ++i)
    if (shapes[i].is_rule) rule_at = i;
  for (size_t i = 0; i < shapes.size(); ++i) {
    if (i >= top && i != rule_at) continue;
    apply(shapes[i].shape);
    double us = 0.0;
    r = time_shape(3 * launches_per_shape, &us);
    if (r != KVD_OK) { apply(before); return r; }
    if (us < shapes[i].us) shapes[i].us = us;
  }
  const double rule_us = shapes[rule_at].us;
  size_t best = rule_at;
  for (size_t i = 0; i < top; ++i)
    if (shapes[i].us < 0.985 * rule_us && shapes[i].us < shapes[best].us) best = i;
  apply(shapes[best].shape);
  if (chosen_shape) {
    chosen_shape[0] = shapes[best].shape.passes; chosen_shape[1] = shapes[best].shape.n_score;
    chosen_shape[2] = shapes[best].shape.splits; chosen_shape[3] = shapes[best].shape.groups;
  }
  if (us_chosen) *us_chosen = (float)shapes[best].us;
  if (us_rule) *us_rule = (float)rule_us;
  return KVD_OK;
}

int kvd_step_form(const kvd_ctx* ctx) {
  if (!ctx) return KVD_ERR_ARG;
  return ctx->single_launch ? -1 : ctx->MB;
}

int kvd_set_wait_limit_us(kvd_ctx* ctx, int64_t microseconds) {
  if (!ctx || microseconds < 0) return KVD_ERR_ARG;
  ctx->wait_limit_ticks = microseconds * 100;        // the GPU wall clock runs at 100 MHz
  return KVD_OK;
}

int kvd_step_timeline(kvd_ctx* ctx, int64_t* host_records, int32_t capacity, int32_t* n_workgroups) {
  if (!ctx || !host_records || !n_workgroups || capacity < 0) return KVD_ERR_ARG;
  if (!ctx->single_launch || ctx->tl_workgroups == 0) return KVD_ERR_STATE;
  HIP_TRY(ctx, hipDeviceSynchronize());
  *n_workgroups = ctx->tl_workgroups;
  int n = ctx->tl_workgroups < capacity ? ctx->tl_workgroups : capacity;
  if (n > KVD_TIMELINE_MAX) n = KVD_TIMELINE_MAX;
  HIP_TRY(ctx, hipMemcpy(host_records, ctx->d_timeline, (size_t)n * 5 * sizeof(int64_t), hipMemcpyDeviceToHost));
  return KVD_OK;
}

int kvd_get_stats(kvd_ctx* ctx, kvd_stats* host_out) {
  if (!ctx || !host_out) return KVD_ERR_ARG;
  unsigned long long raw[4] = {0, 0, 0, 0};
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(raw, ctx->d_stats, sizeof(raw), hipMemcpyDeviceToHost));
  memset(host_out, 0, sizeof(*host_out));
  host_out->steps = ctx->n_steps;
  host_out->hits = raw[0];
  host_out->misses = raw[1];
  host_out->evictions = raw[2];
  host_out->gathered_bytes = raw[1] * (uint64_t)ctx->page_bytes;
  host_out->ms_score = ctx->ms_score;
  host_out->ms_select_resolve = ctx->ms_select_resolve;
  host_out->ms_gather = ctx->ms_gather;
  host_out->ms_attend = ctx->ms_attend;
  host_out->ms_merge = ctx->ms_merge;
  host_out->ms_total = ctx->ms_total;
  host_out->profiled_steps = ctx->profiled_steps;
  if (*ctx->error_host != 0) return KVD_ERR_STATE;
  return KVD_OK;
}

int kvd_reset_stats(kvd_ctx* ctx) {
  if (!ctx) return KVD_ERR_ARG;
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemset(ctx->d_stats, 0, 4 * sizeof(unsigned long long)));
  ctx->n_steps = 0;
  ctx->ms_score = ctx->ms_select_resolve = ctx->ms_gather = ctx->ms_attend = ctx->ms_merge = ctx->ms_total = 0.0;
  ctx->profiled_steps = 0;
  return KVD_OK;
}

}  // extern "C"
