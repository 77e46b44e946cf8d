// Host-side internals of libkvd: the context and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/kvd.h"

constexpr int KVD_MAX_GROUP = 8;        // G = Hq / Hkv
constexpr int KVD_MAX_TOPK = 2048;      // k
constexpr int KVD_MAX_CAPACITY = 65536; // Cmax
constexpr int KVD_FAST_MAX_PAGES = 16384;    // register-resident selection: 1024 threads x 16 pages
constexpr int KVD_FAST_MAX_CAPACITY = 4096; // register-resident directory scan: 1024 threads x 4 slots
constexpr int KVD_MAX_PAGE = 256;       // P
constexpr int KVD_MAX_MICRO = 16;       // micro-batches per step
constexpr int KVD_PIPE_STREAMS = 3;      // side streams a step may spread its micro-batches over
constexpr int KVD_LAYER_LANES = 2;       // layers kvd_step_layers keeps in flight on streams as chains of kernels (three and four measured no faster)
constexpr int KVD_MAX_SETS = 8;          // sets of per-step scratch: the layers one launch of the one-launch step can cover
constexpr int KVD_MAX_SPLITS = 64;      // attention split-K factor
constexpr int KVD_MAX_CENTROIDS = 8192;   // centroids per unit of the hierarchical index (16-bit cluster numbers, <= 65535 pages each)
constexpr int KVD_TIMELINE_MAX = 1 << 16; // workgroups of a single-launch step whose times can be recorded

namespace kvd {
struct FastArgs;
struct AttnArgs;
}  // namespace kvd

// Launch shape of the one-launch step: passes of 64 pages per scoring wave and chunk, persistent
// scoring workgroups (per group), attention splits per unit, groups of units pipelined through the
// launch one behind the other.
struct kvd_shape { int passes, n_score, splits, groups; };

// The per-step scratch of one layer-step in flight (the d_* fields of the context of the same names).
struct kvd_scratch {
  float* scores;
  int32_t *sel_pages, *sel_slots, *hit_mask, *evicted, *counts, *miss_list, *miss_count;
  float *part_acc, *part_ml;
  int32_t *attn_ticket, *score_done;
  unsigned long long* sel_entry;
};

struct kvd_ctx {
  kvd_config cfg;
  int L, B, Hq, Hkv, G, D, P, NP, k, Cmax, Lp, U, MB, S;
  int S1;                  // attention split-K factor of the one-launch step as kvd_create chose it (S: of the stand-alone kernel)
  int S1_max;              // the largest split factor the partials were allocated for
  kvd_shape shape[2];      // launch shape of the one-launch step as set or calibrated, 0 = left to the rule:
                           // [0] launches of one layer (kvd_step), [1] launches of several layers (kvd_step_layers)
  int step_threads;        // workgroup size of the one-launch step: one per CU; 512 (256 registers per lane) or 1024 (128 registers)
  int Nc;                  // centroids per unit of the hierarchical index, 0 = flat page index
  int bf16;
  int score_blocks;        // target number of blocks of a scoring launch
  int generic_select;      // force the size-agnostic select / resolve kernels (testing)
  int fuse_merge;          // attention: last split workgroup merges (1) or a second kernel does (0)
  int single_launch;       // kvd_step runs as one kernel launch
  int tiled;               // slot layout (kvd_tile_layout.h): 0 natural, 1 16-token tiles (page size a multiple of 16), 2 packed (pages of 4 or 8 tokens)
  float scale;
  size_t page_bytes;

  // borrowed
  void* summaries;
  void* centroids;          // [L][U][Nc][D] kv dtype
  int32_t* cluster_start;   // [L][U][Nc+1]
  int32_t* cluster_pages;   // [L][U][NP] pages of every cluster, ascending
  const char* store_dev;    // device-visible address of the pinned host store
  const char* store_host;   // the same store as the host addresses it
  char* pool;

  // owned, device
  int32_t* d_capacity;      // [L][U]
  int32_t* d_seq_len;       // [B]
  int32_t* d_page_to_slot;  // [L][U][NP]   -1 = not resident
  int32_t* d_slot_page;     // [L][U][Cmax] -1 = free
  int32_t* d_slot_stamp;    // [L][U][Cmax]
  int32_t* d_resident;      // [L][U]
  int32_t* d_page_cluster;  // [L][U][NP] cluster of every page (-1 = none); hierarchical index only
  float* d_scores;          // [U][NP]
  const float* last_scores; // where the scores of the most recent scoring went (d_scores or the caller's buffer)
  int32_t* d_sel_pages;     // [U][k]
  int32_t* d_sel_slots;     // [U][k]
  int32_t* d_hit_mask;      // [U][k]
  int32_t* d_evicted;       // [U][k]
  int32_t* d_counts;        // [U][3]
  int32_t* d_miss_list;     // [U][k][2]  (page, slot)
  int32_t* d_miss_count;    // [U]
  float* d_part_acc;        // [U][S][G][D]
  float* d_part_ml;         // [U][S][G][2]  (max in log2 units, sum)
  int32_t* d_attn_ticket;   // [U] arrival counter of the attention splits, zero between launches
  int32_t* d_score_done;    // [U][32] single-launch step: scoring waves arrived (one 128-byte line per unit), zero between launches
  unsigned long long* d_sel_entry;  // [U][k] single-launch step: the selection as its attention workgroups read it (published bit, slot, page); zero between launches
  unsigned long long* d_stats;  // hits, misses, evictions
  // kvd_step_layers keeps several layers in flight, each with its own set of the per-step scratch
  // above: the d_* fields hold set `cur_set`, the others wait in `sets` (contexts of two layers
  // and more; sets[cur_set] itself is stale)
  kvd_scratch sets[KVD_MAX_SETS];
  int n_sets, cur_set;

  // owned, host
  int32_t* h_capacity;      // [L][U]
  int32_t* h_seq_len;       // [B]
  hipStream_t side[KVD_PIPE_STREAMS];   // pipeline streams 1.. (stream 0 is the caller's)
  hipEvent_t ev_fork;
  hipEvent_t ev_score[KVD_MAX_MICRO];   // scoring of micro-batch i has finished
  hipEvent_t ev_done[KVD_MAX_MICRO];    // micro-batch i has finished
  hipEvent_t ev_prof[12];
  int32_t* error_host;      // pinned word the single-launch step raises when one of its waits runs out
  int32_t* error_dev;       // the same word as the GPU addresses it
  long long wait_limit_ticks;   // bound of every in-kernel wait, in ticks of the 100 MHz wall clock
  int n_cus;                // compute units of the device
  long long* d_timeline;    // [KVD_TIMELINE_MAX][5] per-workgroup record of the last single-launch step
  int tl_workgroups;        // workgroups of that launch
  // third tier (borrowed) and what kvd_step_tiered hands across the host boundary
  kvd_tier* tier;
  const char* tier_pool_dev;  // the tier's pool as the GPU addresses it
  int32_t* h_miss_list;       // pinned [U][k][2]
  int32_t* h_miss_count;      // pinned [U]
  int64_t* h_src_offset;      // pinned [U][k]
  int64_t* d_src_offset;      // [U][k]
  int wait_timeouts;          // one-launch steps that gave up waiting (each one switched the context to the chain of kernels)
  int profiling;
  int last_hip;
  uint64_t n_steps;
  double ms_score, ms_select_resolve, ms_gather, ms_attend, ms_merge, ms_total;
  uint64_t profiled_steps;
};

// Kernel launchers.  u0/u1 bound the units [u0, u1) of the layer that the launch covers.
hipError_t kvd_launch_score(kvd_ctx* c, int layer, const void* q, float* scores, int u0, int u1, hipStream_t s);
hipError_t kvd_launch_select(kvd_ctx* c, const float* scores, int32_t* sel_pages, int u0, int u1, hipStream_t s);
hipError_t kvd_launch_resolve(kvd_ctx* c, int layer, int step, const int32_t* sel_pages, int32_t* sel_slots,
                              int32_t* hit_mask, int32_t* evicted, int32_t* counts, int u0, int u1, hipStream_t s);
bool kvd_fast_path_ok(const kvd_ctx* c);
hipError_t kvd_launch_select_resolve(kvd_ctx* c, int layer, int step, bool do_select, bool do_resolve, bool do_gather,
                                     const float* scores, int32_t* sel_pages, int32_t* sel_slots, int32_t* hit_mask,
                                     int32_t* evicted, int32_t* counts, int u0, int u1, hipStream_t s);
kvd::FastArgs kvd_fast_args(kvd_ctx* c, int layer, int step, bool do_gather, const float* scores, int32_t* sel_pages,
                            int32_t* sel_slots, int32_t* hit_mask, int32_t* evicted, int32_t* counts, int u0);
kvd::AttnArgs kvd_attn_args(kvd_ctx* c, int layer, const void* q, const int32_t* sel_pages, const int32_t* sel_slots,
                            float* out, float* lse, int u0);
// Copies the missed pages of units [u0, u1) into their slots: from the pinned host store, or, with
// src_base / src_offset ([U][k] byte offsets, -1 = skip), from wherever the caller says each one is.
hipError_t kvd_launch_gather(kvd_ctx* c, int layer, int u0, int u1, hipStream_t s, const char* src_base = nullptr,
                             const int64_t* src_offset = nullptr);
// kvd_tier.hip
const kvd_tier_config* kvd_tier_config_of(const kvd_tier* t);
void* kvd_tier_pool_of(const kvd_tier* t);
hipError_t kvd_launch_attend(kvd_ctx* c, int layer, const void* q, const int32_t* sel_pages,
                             const int32_t* sel_slots, float* out, float* lse, int u0, int u1, hipStream_t s,
                             hipEvent_t between = nullptr);   // `between`: recorded after the attention kernel, before the merge
// The whole step as one launch (kvd_step.hip); usable when kvd_single_launch_ok.
bool kvd_single_launch_ok(const kvd_ctx* c);
// The shape a launch takes: `want` (default: what the context holds for that kind of launch) with
// its zeros filled in by the rule and the scoring workgroups capped at the number of chunks.
kvd_shape kvd_step_shape(const kvd_ctx* c, int multi_layer, const kvd_shape* want = nullptr);
bool kvd_step_shape_ok(const kvd_ctx* c, const kvd_shape& effective);
// Layers [layer, layer + n_layers) of one decode step in one launch, layer `layer + i` in scratch set i
// (q / out / lse: the layers one after another); n_layers == 1: the context's current set.
hipError_t kvd_launch_step(kvd_ctx* c, int layer, int n_layers, int step, const void* q, float* out, float* lse, hipStream_t s);
// Scratch set i of the context, wherever its pointers currently are (kvd_api.hip).
kvd_scratch kvd_scratch_set(const kvd_ctx* c, int i);
hipError_t kvd_launch_refill(kvd_ctx* c, int layer, hipStream_t s);
hipError_t kvd_launch_build_summaries(kvd_ctx* c, int layer, hipStream_t s);
bool kvd_centroid_mode(const kvd_ctx* c);
hipError_t kvd_prepare_cluster_select(void);
hipError_t kvd_launch_cluster_select(kvd_ctx* c, int layer, const float* scores, int32_t* sel_pages, int u0, int u1,
                                     hipStream_t s);
hipError_t kvd_launch_cluster_inverse(kvd_ctx* c, int layer, hipStream_t s);
hipError_t kvd_run_build_centroids(kvd_ctx* c, int layer, int iterations, int32_t* assign_trace, hipStream_t s);
hipError_t kvd_launch_append(kvd_ctx* c, int layer, const void* k_new, const void* v_new, hipStream_t s);
hipError_t kvd_launch_advance(kvd_ctx* c, hipStream_t s);
hipError_t kvd_launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t s);
