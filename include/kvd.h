/*
 * kvd.h — C ABI of libkvd: the per-layer decode hot path of KVDrive-style
 * offloaded sparse attention on AMD MI355X (gfx950).
 *
 * One decode step of one layer is the three-stage workflow the paper states in
 * "KV Cache Offloading" (Background) and "System Overview":
 *   (1) select the critical KV pages through an index held in GPU memory,
 *   (2) fetch the selected pages that are not resident from host memory,
 *   (3) run sparse attention over resident + fetched pages.
 * The index is the mean key of each page (System Overview); the in-GPU cache is
 * the window of recently critical pages of "Attention-Based Cache Management",
 * with LRU replacement or the paper's lookahead eviction (kvd_policy); stage (2)
 * moves only out-of-cache pages ("Performance Analysis via Roofline Model").
 *
 * Notation: L layers, B sequences, Hq query heads, Hkv KV heads, G = Hq/Hkv,
 * D = head_dim = 128, P tokens per page, NP pages per sequence, k pages selected
 * per step, C cache pages per unit.  A *unit* is one (layer, sequence, KV head);
 * u = b*Hkv + h indexes the units of a layer, U = B*Hkv.  KV elements are 2 bytes
 * (fp16 or bf16); page_bytes = 2*P*D*2 (the K page followed by the V page).
 *
 * Conventions
 *   - every function returns KVD_OK (0) or a negative kvd_status; nothing throws;
 *   - "dev" pointers are device (HBM) pointers, "host" pointers are ordinary host
 *     memory, "pinned" is page-locked host memory that the GPU can address;
 *   - data buffers (summaries, host store, slot pool, q, out, selections) belong
 *     to the caller and are only borrowed; the library owns its kvd_ctx (cache
 *     directory, scratch, miss lists, a few side streams, events) until kvd_destroy;
 *   - hot-path calls enqueue work on the caller's hipStream_t (passed as void*,
 *     NULL = the null stream) and return without waiting; outputs are valid once
 *     that stream has been synchronised.  No decision is taken on the host
 *     between stages, so a call sequence can be captured in a HIP graph;
 *   - calls on one kvd_ctx must not overlap in time on different streams.
 */
#ifndef KVD_H
#define KVD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvd_ctx kvd_ctx;

typedef enum {
  KVD_OK = 0,
  KVD_ERR_ARG = -1,      /* NULL / misaligned / not device-addressable pointer, bad index */
  KVD_ERR_SHAPE = -2,    /* inconsistent or unsupported sizes */
  KVD_ERR_CAPACITY = -3, /* k > C for some unit, forced pages > k, warm list > C, tier pool too small for a step */
  KVD_ERR_DTYPE = -4,
  KVD_ERR_HIP = -5,      /* a HIP runtime call failed; see kvd_last_hip_error */
  KVD_ERR_STATE = -6     /* buffers not bound yet, an imported directory breaks its invariants, an in-kernel wait
                            ran out, or a file operation of the third tier failed */
} kvd_status;

typedef enum { KVD_F16 = 0, KVD_BF16 = 1 } kvd_dtype;
/* Which resident pages leave a full window (Cache Management, "Sliding Window w/ Lookahead
 * Eviction"): LRU drops the least recently selected pages; LOOKAHEAD drops the pages with the
 * lowest page score of the current step (equal scores: the higher page index first), the
 * attention-derived importance that is known for every page of the index. */
typedef enum { KVD_EVICT_LRU = 0, KVD_EVICT_LOOKAHEAD = 1 } kvd_policy;

typedef struct {
  int32_t n_layers;        /* L */
  int32_t batch;           /* B */
  int32_t n_q_heads;       /* Hq, a multiple of n_kv_heads, G = Hq/Hkv <= 8 */
  int32_t n_kv_heads;      /* Hkv */
  int32_t head_dim;        /* D, must be 128 */
  int32_t page_size;       /* P, 1..256 */
  int32_t max_pages;       /* NP: pages allocated per sequence in every buffer */
  int32_t topk_pages;      /* k = token budget / P */
  int32_t sink_pages;      /* first pages of a sequence, always selected, counted inside k */
  int32_t recent_pages;    /* last valid pages of a sequence, always selected, counted inside k
                              (Experiment, Baselines: sink and local tokens stay on the GPU) */
  int32_t kv_dtype;        /* kvd_dtype: element type of q, summaries, host store and slot pool */
  int32_t policy;          /* kvd_policy */
  float   softmax_scale;   /* multiplies q.k in scoring and attention; 0 means 1/sqrt(D) */
  int32_t capacity_max;    /* Cmax: slots allocated per unit in the slot pool */
  const int32_t* capacity; /* host, [L*U] pages per unit (per-layer, per-head window sizes, the
                              run-time side of "2D Window Scaling"); NULL = capacity_max everywhere.
                              Copied by kvd_create. */
  int32_t physical_layers; /* layers present in the host store; layer l reads store layer
                              l % physical_layers.  0 means n_layers. */
  int32_t micro_batches;   /* how kvd_step overlaps selection, fetch and attention ("SFC Disaggregation"):
                              -1 = the whole step as one launch in which every (sequence, KV head) unit
                                   moves through the stages on its own, synchronised by counters and
                                   published words in device memory (needs a page size that is a multiple of
                                   16, or 4, or 8; max_pages <= 16384; capacity_max <= 4096; other shapes run
                                   as for 1).  A workgroup of that
                                   launch only ever waits for workgroups with a lower index, and the form
                                   relies on the GPU starting the workgroups of a one-dimensional grid in
                                   index order (what a waiting workgroup waits for has then started and
                                   itself waits only for still lower ones: the launch cannot lock up, and
                                   neither can two such launches on two streams, whose chains of waits stay
                                   inside each launch).  The programming model does not promise that order,
                                   so every wait is bounded (kvd_set_wait_limit_us); should one run out, the
                                   library recovers by itself as described there;
                              0  = chosen by the library: the one launch where it can run (with units of
                                   more than 8192 pages only from 24 units on), else as for 1;
                              1  = one chain of kernels on the caller's stream, no overlap;
                              n >= 2 = the B sequences are split into n groups, each running
                                   select -> fetch -> attend as its own chain on one of the library's
                                   streams, so the fetch of one group overlaps the kernels of the others. */
  int32_t attn_splits;     /* split-K factor of the attention kernel; 0 = chosen by the library */
  int32_t index_centroids; /* Nc: 0 = selection scores every page summary (flat index); > 0 = hierarchical
                              index (System Overview: the page means form higher-level centroids): the page
                              summaries of a unit are grouped into Nc clusters by k-means, selection scores
                              the Nc centroids and takes whole clusters, best first, until k pages are used
                              (the first cluster that does not fit gives its lowest pages; sink / recent pages
                              are in first and do not count as members).  Nc <= 8192, Nc <= max_pages <= 16384;
                              kvd_step runs in any of its forms.  Under KVD_EVICT_LOOKAHEAD the score
                              of a resident page is the score of its cluster (a page of no cluster leaves
                              first; pages of one cluster: the higher page first). */
  int32_t lookahead_pool;  /* M, the look-ahead candidate pool of KVD_EVICT_LOOKAHEAD (Experiment, "Generality of
                              Eviction Policy": M = 2560 entries for a budget of 2048), in pages; 0 = every scored
                              page.  The M best-scoring pages of a step (score descending, ties to the lower page)
                              are the candidates for reuse: resident pages outside them leave first, least
                              recently selected first (smallest (stamp, page)); pool pages only after those,
                              lowest score first.  M >= the valid pages of a sequence is the policy without a
                              pool; M == topk_pages (without sink / recent pages) is LRU. */
} kvd_config;

typedef struct {
  uint64_t steps;          /* layer-steps executed by kvd_step / kvd_cache_resolve */
  uint64_t hits;           /* selected pages found resident */
  uint64_t misses;         /* selected pages fetched from the host store */
  uint64_t evictions;      /* pages dropped from the window */
  uint64_t gathered_bytes; /* misses * page_bytes */
  /* filled only while profiling is on (kvd_set_profiling): accumulated milliseconds per kernel,
     from HIP events recorded around each launch on the stream it runs on */
  double ms_score;          /* scoring kernel */
  double ms_select_resolve; /* selection + directory update; on the fused path also the fetch */
  double ms_gather;         /* separate fetch kernel (size-agnostic path only) */
  double ms_attend;         /* attention kernel */
  double ms_merge;          /* merge of the attention splits */
  double ms_total;
  uint64_t profiled_steps;
} kvd_stats;

/* ---- life cycle ------------------------------------------------------------------------- */

/* Validates cfg, allocates the directory (all units empty) and scratch on the current HIP
 * device.  *out receives the context.  KVD_ERR_SHAPE / KVD_ERR_CAPACITY / KVD_ERR_DTYPE on a
 * bad configuration (nothing is allocated then), KVD_ERR_HIP if an allocation fails. */
int kvd_create(const kvd_config* cfg, kvd_ctx** out);
int kvd_destroy(kvd_ctx* ctx);

const char* kvd_strerror(int status);
int kvd_last_hip_error(const kvd_ctx* ctx);   /* hipError_t of the last failed runtime call */
int kvd_abi_version(void);

/* ---- buffers (borrowed) ------------------------------------------------------------------ */

/* Index: mean key of each page, dev, [L][B][Hkv][NP][D] kv_dtype, 16-byte aligned. */
int kvd_bind_summaries(kvd_ctx* ctx, void* dev_summaries);
/* Paged KV store in pinned host memory, [Lp][B][Hkv][NP][2][P][D] kv_dtype (K page, then V
 * page).  KVD_ERR_ARG if the GPU cannot address the pointer. */
int kvd_bind_host_store(kvd_ctx* ctx, const void* pinned_store);
/* GPU cache tier, dev, [L][B][Hkv][Cmax] slots of page_bytes each, 16-byte aligned.  Contents are
 * managed by the library: which page sits in which slot is the directory's business, and inside a
 * slot the page is stored in the order the attention kernel reads it (pages of a multiple of 16
 * tokens: 16-token tiles of MFMA-operand-ready K and transposed V; pages of 4 or 8 tokens: the same
 * operands packed per page, 16 / P selected pages forming one tile; otherwise K[P][D] then V[P][D]). */
int kvd_bind_slot_pool(kvd_ctx* ctx, void* dev_pool);
/* Valid tokens per sequence, host [B], each in 1..NP*P.  Default: NP*P.  Synchronous. */
int kvd_set_seq_lens(kvd_ctx* ctx, const int32_t* host_seq_len);

/* ---- set-up helpers (not on the hot path) ------------------------------------------------- */

/* Builds the index of one layer from the host store: summary[p][d] = mean over the valid tokens
 * of page p of K[token][d], accumulated in fp64 in token order and rounded once to kv_dtype
 * (System Overview: the mean key of each page is its representative).  Enqueued on stream. */
int kvd_build_summaries(kvd_ctx* ctx, int32_t layer, void* stream);

/* Empties the directory of every layer (cold cache).  Synchronous. */
int kvd_cache_reset(kvd_ctx* ctx);
/* Replaces one layer's cache content: unit u becomes resident with pages
 * host_pages[off_u .. off_u+host_counts[u]) (off_u = sum of earlier counts), stamp -1, and the
 * page data is copied from the host store.  KVD_ERR_CAPACITY if a count exceeds the unit's
 * capacity, KVD_ERR_ARG on a page out of range or repeated.  Synchronous. */
int kvd_cache_warm(kvd_ctx* ctx, int32_t layer, const int32_t* host_pages, const int32_t* host_counts);
/* Directory of one layer as flat arrays, host, [U][Cmax] each: page in the slot (-1 = free) and
 * the step at which it was last selected.  Synchronous. */
int kvd_cache_export(kvd_ctx* ctx, int32_t layer, int32_t* host_slot_page, int32_t* host_slot_stamp);
/* Installs a directory (same arrays as export) and refills the named slots from the host store.
 * KVD_ERR_STATE if a page repeats inside a unit, is out of range, or a slot >= the unit's
 * capacity is occupied; the cache is left unchanged then.  Synchronous. */
int kvd_cache_import(kvd_ctx* ctx, int32_t layer, const int32_t* host_slot_page, const int32_t* host_slot_stamp);

/* ---- hot path: each stage alone (all pointers dev) ----------------------------------------- */

/* Stage 1, selection (Background: the query is multiplied with the index and the Top-K kept).
 *   q          [B][Hq][D] kv_dtype.  The G query heads of a KV head are mean-pooled in fp32.
 *   sel_pages  [B][Hkv][k] int32 out: the k pages with the largest
 *              score = scale * pooled_q . summary, ties to the lower page; sink/recent pages
 *              always included; ascending page order; padded with -1 when a sequence has fewer
 *              than k valid pages.
 *   scores     [B][Hkv][NP] fp32 out, or NULL.
 * With the hierarchical index (index_centroids = Nc > 0) the centroids are scored instead and the
 * pages come from whole clusters taken best first (see kvd_config.index_centroids); `scores` must
 * still hold B*Hkv*NP floats and receives the cluster scores packed as [B][Hkv][Nc]. */
int kvd_score_select(kvd_ctx* ctx, int32_t layer, const void* q, int32_t* sel_pages, float* scores, void* stream);

/* Stage 2, cache lookup and fetch (Cache Management; Roofline section: only out-of-cache pages move).
 *   sel_pages  [B][Hkv][k] from stage 1.
 *   sel_slots  [B][Hkv][k] int32 out: slot of each selected page (-1 where sel_pages is -1).
 *   hit_mask   [B][Hkv][k] int32 out or NULL: 1 = was resident, 0 = fetched.
 *   evicted    [B][Hkv][k] int32 out or NULL: pages dropped in this step, -1 padded, unordered.
 *   counts     [B][Hkv][3] int32 out or NULL: hits, misses, evictions.
 * Hits are re-stamped with `step`; misses take free slots first, then the slots of the resident
 * pages, not selected in this step, with the smallest (stamp, page) — under KVD_EVICT_LOOKAHEAD
 * with the smallest (score, -page), read from where the most recent kvd_score_select of this
 * context left its scores (KVD_ERR_STATE if there was none).  `step` must not decrease for a
 * layer.  With do_gather != 0 the missed pages are then copied from the host store into their
 * slots on `stream`.  With do_gather == 0 only the directory changes (slot contents are
 * stale).  sel_pages must hold distinct pages in ascending order, as stage 1 writes them. */
int kvd_cache_resolve(kvd_ctx* ctx, int32_t layer, int32_t step, const int32_t* sel_pages, int32_t* sel_slots,
                      int32_t* hit_mask, int32_t* evicted, int32_t* counts, int32_t do_gather, void* stream);

/* Stage 3, sparse attention (System Overview: attention over resident and fetched entries).
 *   out [B][Hq][D] fp32 = softmax(scale * q K_sel^T) V_sel over the valid tokens of the selected
 *   pages, read from the slot pool through sel_slots; fp32 accumulation, online softmax,
 *   split over the selected pages and merged by log-sum-exp.
 *   lse [B][Hq] fp32 out or NULL: log sum exp of the scaled logits. */
int kvd_sparse_decode_attn(kvd_ctx* ctx, int32_t layer, const void* q, const int32_t* sel_pages,
                           const int32_t* sel_slots, float* out, float* lse, void* stream);

/* Stage 3 for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same attention as kvd_sparse_decode_attn, without a
 * context: the call takes everything it needs as arguments and neither it nor anything it calls
 * allocates or frees (no hipMalloc, hipFree or allocating library routine).  Its split partials and
 * arrival tickets live in one 8 MiB array of device memory that is part of the library's code object:
 * every GPU the library runs on holds its own copy from the moment the library is loaded there until
 * the process ends.
 *   q          dev [B][Hq][D] kv_dtype, 16-byte aligned (D = 128)
 *   slot_pool  dev [B][Hkv][Cmax] slots of 2*P*D*2 bytes, 16-byte aligned: one layer of a pool in the
 *              library's slot order, i.e. as kvd_cache_resolve / kvd_step of a context of the same
 *              P and Cmax filled it (layer l of that pool starts l*B*Hkv*Cmax slots in)
 *   sel_pages, sel_slots  dev [B][Hkv][k] int32, as stages 1 and 2 write them (-1 = padding)
 *   seq_len    dev [B] int32 valid tokens per sequence
 *   out        dev [B][Hq][D] fp32;  lse  dev [B][Hq] fp32 or NULL
 *   softmax_scale  0 means 1/sqrt(D);  attn_splits  split-K factor, 0 = chosen as kvd_create does.
 * Limits: those of kvd_config (G <= 8, P <= 256, k <= 2048, B*Hkv <= 65535), and
 * B*Hkv*(4 + splits*G*520) bytes (each part rounded up to 256) must fit the 8 MiB array:
 * KVD_ERR_CAPACITY otherwise, nothing is enqueued then.  KVD_ERR_ARG / KVD_ERR_SHAPE / KVD_ERR_DTYPE
 * as kvd_create and kvd_sparse_decode_attn; KVD_ERR_HIP if the array's address cannot be obtained
 * or a launch fails.  The first call on a GPU looks up that GPU's copy of the array
 * (hipGetSymbolAddress) and must therefore come before any graph capture.  Enqueued on `stream`
 * (a fill kernel that zeroes the tickets, then the attention kernel).  Every call on one GPU uses
 * that GPU's one array: calls that overlap in time on one GPU (different streams, or graphs
 * replayed concurrently) race and give wrong results; calls on one stream, one after another, are safe. */
int kvd_sparse_decode_attn_noalloc(const void* q, const void* slot_pool, const int32_t* sel_pages,
                                   const int32_t* sel_slots, const int32_t* seq_len, float* out, float* lse,
                                   int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t page_size,
                                   int32_t topk_pages, int32_t capacity_max, int32_t kv_dtype, float softmax_scale,
                                   int32_t attn_splits, void* stream);

/* ---- hierarchical index ------------------------------------------------------------------------ */

/* Buffers of the hierarchical index (index_centroids = Nc > 0), all device memory owned by the caller:
 *   dev_centroids      [L][B][Hkv][Nc][D] kv_dtype, 16-byte aligned
 *   dev_cluster_start  [L][B][Hkv][Nc+1] int32: cluster c owns entries [start[c], start[c+1]) of
 *   dev_cluster_pages  [L][B][Hkv][NP] int32: the pages of every cluster, ascending inside a cluster. */
int kvd_bind_centroids(kvd_ctx* ctx, void* dev_centroids, int32_t* dev_cluster_start, int32_t* dev_cluster_pages);
/* Set-up helper: builds one layer's hierarchical index from its page summaries (kvd_build_summaries
 * first) by Lloyd's k-means in fp64: initial centroids = the pages at positions
 * floor((c + 1/2) * valid_pages / Nc); `iterations` (1..64) rounds of {nearest centroid by squared
 * Euclidean distance, ties to the lower centroid; centroid = mean of its pages' summaries summed in
 * ascending page order, an empty cluster keeps its centroid}; the stored centroid is rounded once to
 * kv_dtype; the cluster lists are those of the last round.  Covers the pages valid at the time of the
 * call.  dev_assign_trace: device [iterations][B][Hkv][NP] int32 receiving every round's assignment,
 * or NULL.  Allocates temporary device memory and waits for `stream`. */
int kvd_build_centroids(kvd_ctx* ctx, int32_t layer, int32_t iterations, int32_t* dev_assign_trace, void* stream);
/* After the caller has written a layer's cluster lists itself (instead of kvd_build_centroids):
 * recomputes the library's page -> cluster table from them, which lookahead eviction reads.  Enqueued
 * on `stream`.  KVD_ERR_STATE without bound centroids. */
int kvd_refresh_clusters(kvd_ctx* ctx, int32_t layer, void* stream);

/* ---- growth of the KV store during decoding ------------------------------------------------ */

/* Appends the key and value of the token just decoded (Background, "KV Cache Basics": each decoding
 * step appends new key and value vectors) for one layer, at position seq_len[b] of every sequence:
 *   k_new, v_new  device, [B][Hkv][D] kv_dtype, 16-byte aligned.
 * The token is written into the pinned host store (the library writes to the buffer given to
 * kvd_bind_host_store), into the page's slot if the page is resident, and the page's index entry
 * becomes the mean over its valid tokens including the new one.  seq_len does not change: call
 * kvd_advance once every layer has appended.  Enqueued on `stream`; order it after the layer's
 * kvd_step of this decode step and before the next one.  With a tier bound (kvd_bind_tier) the
 * call then waits for `stream` and carries the token's two rows from the host store into the
 * backing file and, where the page's extent is pooled, into the pool (the host store holds the
 * growing pages; the file stays the full backing store).
 * KVD_ERR_SHAPE when a sequence already fills max_pages * page_size tokens; KVD_ERR_STATE when
 * buffers are not bound or physical_layers < n_layers (layers sharing a stored layer cannot append). */
int kvd_append_kv(kvd_ctx* ctx, int32_t layer, const void* k_new, const void* v_new, void* stream);
/* seq_len[b] += 1 for every sequence (device copy on `stream`, host copy at once). */
int kvd_advance(kvd_ctx* ctx, void* stream);

/* ---- hot path: the whole layer-step -------------------------------------------------------- */

/* Stages 1-3 for one layer.  With micro_batches > 1 the groups of sequences run as separate
 * chains on the library's streams (forked from and joined back into `stream`), so that the
 * host-link fetch of one group overlaps the kernels of the others (SFC Disaggregation); otherwise
 * everything is enqueued on `stream`.
 *   q [B][Hq][D] kv_dtype, out [B][Hq][D] fp32, lse [B][Hq] fp32 or NULL. */
int kvd_step(kvd_ctx* ctx, int32_t layer, int32_t step, const void* q, float* out, float* lse, void* stream);

/* The same layer-step for the consecutive layers [layer0, layer0 + n_layers) of one decode step,
 * for a caller that has all their queries at hand (a benchmark, or a model that computes the
 * queries of several layers before their attention; layers whose query depends on the previous
 * layer's attention output are stepped one by one with kvd_step).  Every layer has its own cache
 * directory and slots, so the results are those of the layers stepped one after another; what
 * changes is that the layers overlap (SFC Disaggregation applied across layers):
 *   - where the step runs as one launch, up to 8 layers share a launch whose workgroups are ordered
 *     so that layer l+1 is scored while layer l is being selected and its missed pages are fetched,
 *     and layer l is attended while layer l+1 is selected; everything stays on `stream`;
 *   - where it runs as a chain of kernels, two layers are kept in flight: layers alternate between
 *     `stream` and one of the library's streams (forked from and joined back into `stream` with
 *     events), each with its own per-step scratch.  Groups of sequences (micro_batches > 1) are
 *     not formed here.
 * With profiling on, or in a context of one layer, the layers simply run one after another on `stream`.
 *   q_layers [n_layers][B][Hq][D] kv_dtype, out_layers [n_layers][B][Hq][D] fp32,
 *   lse_layers [n_layers][B][Hq] fp32 or NULL (all device, 16-byte aligned).
 * The call can be captured into a HIP graph from `stream`.  kvd_step_trace afterwards reports the
 * last of the layers.  Errors as kvd_step; KVD_ERR_ARG when the layer range leaves the context's. */
int kvd_step_layers(kvd_ctx* ctx, int32_t layer0, int32_t n_layers, int32_t step, const void* q_layers,
                    float* out_layers, float* lse_layers, void* stream);

/* Copies what the last kvd_step left behind into caller buffers (all dev, any may be NULL),
 * asynchronously on `stream` (which must be ordered after that kvd_step): sel_pages, sel_slots,
 * hit_mask, evicted [B][Hkv][k] int32, counts [B][Hkv][3] int32, scores [B][Hkv][NP] fp32. */
int kvd_step_trace(kvd_ctx* ctx, int32_t* sel_pages, int32_t* sel_slots, int32_t* hit_mask, int32_t* evicted,
                   int32_t* counts, float* scores, void* stream);

/* ---- third tier: backing file on SSD, pool of extents in host DRAM --------------------------- */
/*
 * "Cross-tier Synergistic Storage": the backing file holds every page (the full backing store);
 * host DRAM holds a bounded pool; the GPU window is unchanged.
 *
 * Layout of the file ("SSD-Aware Layout Planning").  An *extent* is a contiguous block of
 * extent_pages pages.  Every {layer, head} unit has a segment of its own, NE = ceil(NP /
 * extent_pages) extents long, segments in (physical layer, unit) order; extent number
 * x = ((layer * U) + unit) * NE + e starts at byte x * extent_pages * page_bytes.  Inside a
 * segment page p sits at place position[unit][p] (a permutation of 0..NP-1; places NP.. of the last
 * extent are padding): pages that are attended together — one cluster of the hierarchical index —
 * are neighbours (kvd_layout_from_clusters), else page order.  A page keeps the host store's
 * natural layout (K[P][D] then V[P][D]).
 *
 * Per step ("Parallel Sparse Synchronization", (b) block-level sparse fetching and (c)
 * hierarchical transfer): the pages that missed in the GPU window are mapped to extents; extents
 * already in the DRAM pool are hits; the others are read whole from the file, runs of neighbouring
 * extents of one segment as one read of at most max_run_extents extents, queue_depth reads in
 * flight; reads land directly in the pool (a fixed set of pinned buffers, allocated once by the
 * caller), from where the GPU copies the missed pages into their slots.  The pool is replaced LRU by
 * extent: when it overflows, the pooled extents that the current step does not need leave in
 * (step of last use, extent number) order.
 *
 * A kvd_tier is plain host code: it needs no GPU, and its pool may be any host memory (pinned
 * memory when a GPU is to read it).  Calls on one kvd_tier must not overlap in time.
 */
typedef struct kvd_tier kvd_tier;

typedef struct {
  int32_t n_layers;         /* physical layers held by the file */
  int32_t n_units;          /* U = B * Hkv */
  int32_t max_pages;        /* NP */
  int32_t extent_pages;     /* pages per extent, >= 1 */
  int64_t page_bytes;       /* 2 * P * D * 2; extent bytes must be a multiple of 4096 for direct I/O */
  int64_t pool_extents;     /* capacity of the DRAM pool, in extents */
  int32_t queue_depth;      /* reader threads, 1..64 */
  int32_t max_run_extents;  /* longest run of neighbouring extents merged into one read, 1..64 */
  int32_t direct_io;        /* 1: open the file with O_DIRECT if the file system takes it (reads then
                               bypass the page cache), falling back to buffered reads otherwise; see
                               kvd_tier_stats.direct_io for what was taken */
} kvd_tier_config;

typedef struct {
  uint64_t steps;           /* kvd_tier_fetch calls */
  uint64_t pages_requested; /* missed pages handed in */
  uint64_t extents_needed;  /* distinct extents those pages lie in, summed over the calls */
  uint64_t extent_hits;     /* ... found in the pool */
  uint64_t extent_reads;    /* ... read from the file */
  uint64_t extent_evictions;
  uint64_t reads_issued;    /* read calls after merging */
  uint64_t bytes_read;
  double ms_plan;           /* host time spent on lookup, replacement and planning */
  double ms_io;             /* wall time from the first read issued to the last one done */
  int32_t direct_io;        /* 0: buffered reads; 1: O_DIRECT straight into the pool; 2: O_DIRECT into one
                               aligned staging buffer per reader, copied into the pool from there (taken from the
                               first read on that the file system refuses into the pool's memory) */
} kvd_tier_stats;

/* Opens (creating and sizing it if need be) the backing file and takes `pool_host`, pool_extents *
 * extent_pages * page_bytes bytes of caller-owned host memory, 4096-byte aligned, as the DRAM pool.
 * The layout starts as page order for every unit; the pool starts empty.  KVD_ERR_ARG for NULL
 * pointers, KVD_ERR_SHAPE for sizes out of range, KVD_ERR_STATE if the file cannot be opened or
 * sized (errno is kept: kvd_tier_last_errno). */
int kvd_tier_open(const kvd_tier_config* cfg, const char* path, void* pool_host, kvd_tier** out);
int kvd_tier_close(kvd_tier* tier);
int kvd_tier_last_errno(const kvd_tier* tier);
/* Places of the pages of one physical layer: host_position [U][NP], every row a permutation of
 * 0..NP-1 (KVD_ERR_ARG otherwise).  Set before that layer is written. */
int kvd_tier_set_layout(kvd_tier* tier, int32_t layer, const int32_t* host_position);
/* Set-up helper: writes the pages of one physical layer, host_pages [U][NP][page_bytes] in the host
 * store's order, to their places in the file (buffered writes, then fsync) and drops that layer's
 * extents from the pool. */
int kvd_tier_write_layer(kvd_tier* tier, int32_t layer, const void* host_pages);
/* Growth helper: overwrites nbytes at offset_in_page of one page with host_src, in the file
 * (buffered write; later reads of the file see it) and in the pool's copy if the page's extent is
 * pooled.  offset_in_page + nbytes <= page_bytes. */
int kvd_tier_patch_page(kvd_tier* tier, int32_t layer, int32_t unit, int32_t page, int64_t offset_in_page,
                        const void* host_src, int64_t nbytes);
/* One step of one physical layer.  host_miss_list [U][k][2] (page, slot) and host_miss_count [U] are
 * the GPU window's misses as the resolve stage leaves them (entries with slot < 0 are skipped).
 * On return every needed extent is in the pool and host_src_offset [U][k] holds, for entry j < count
 * of unit u, the byte offset of that page inside the pool (-1 for skipped entries).  Synchronous.
 * KVD_ERR_CAPACITY if the step needs more extents than the pool holds (nothing is changed),
 * KVD_ERR_ARG for a page out of range, KVD_ERR_STATE if a read fails or comes back short. */
int kvd_tier_fetch(kvd_tier* tier, int32_t layer, int32_t step, const int32_t* host_miss_list,
                   const int32_t* host_miss_count, int32_t k, int64_t* host_src_offset);
/* What the last kvd_tier_fetch did.  counts[5]: extents needed, hits, reads, evictions, read calls.
 * runs [cap_runs][2] receives (first extent, number of extents) of the read calls in file order,
 * evicted [cap_evicted] the evicted extents in ascending order (each list cut at its capacity;
 * either may be NULL). */
int kvd_tier_trace(const kvd_tier* tier, int64_t* counts, int64_t* runs, int64_t cap_runs, int64_t* evicted,
                   int64_t cap_evicted);
/* Which extents the pool holds: writes up to cap extent numbers in ascending order, and the number
 * held to *n_pooled. */
int kvd_tier_pooled(const kvd_tier* tier, int64_t* extents, int64_t cap, int64_t* n_pooled);
int kvd_tier_drop_pool(kvd_tier* tier);          /* empties the DRAM pool (the file is untouched) */
int kvd_tier_get_stats(const kvd_tier* tier, kvd_tier_stats* out);
int kvd_tier_reset_stats(kvd_tier* tier);
/* Measurement helper: reads the whole file once, front to back, in reads of max_run_extents extents
 * with queue_depth readers into the pool's memory (the pool is dropped), and reports the rate — what
 * this file, opened this way, gives a purely sequential reader. */
int kvd_tier_sequential_read_gbps(kvd_tier* tier, double* gbps);

/* Semantic-contiguity layout from the bound hierarchical index of `layer`: host_position [U][NP]
 * puts the pages of a unit cluster by cluster (cluster ascending, page ascending within; pages
 * beyond the valid length last).  Synchronises the device.  KVD_ERR_STATE without bound centroids. */
int kvd_layout_from_clusters(kvd_ctx* ctx, int32_t layer, int32_t* host_position);
/* Attaches a tier to the context: kvd_step_tiered then takes missed pages from it.  The tier's pool
 * must be pinned host memory (KVD_ERR_ARG otherwise) and its sizes must match the context's (units,
 * pages, page bytes, physical layers; KVD_ERR_SHAPE otherwise).  The tier stays the caller's and
 * must outlive its use by the context.  NULL detaches. */
int kvd_bind_tier(kvd_ctx* ctx, kvd_tier* tier);
/* kvd_step with the third tier behind the window: score, select and directory update run on the
 * GPU as in kvd_step; the miss lists are then handed to the host (this call waits for them — the
 * host has to issue the reads), kvd_tier_fetch brings the extents into the pool, and the copy of
 * the missed pages from the pool into their slots and the attention are enqueued on `stream`.
 * Outputs are valid once the stream has been synchronised.  The pinned host store is not read.
 * If the tier fails (KVD_ERR_CAPACITY: the step needs more extents than the pool holds;
 * KVD_ERR_STATE: a read failed) no output is produced and the window of `layer` is emptied, since
 * its directory had already been updated for pages that did not arrive. */
int kvd_step_tiered(kvd_ctx* ctx, int32_t layer, int32_t step, const void* q, float* out, float* lse, void* stream);

/* ---- counters ------------------------------------------------------------------------------ */

/* mode 0: off.
 * mode 1: kvd_step runs as a chain of separate kernels, brackets every stage with HIP events on the
 *         stream, waits for the step and adds the stage times to the stats (the step is then
 *         synchronous).
 * mode 2: a single-launch kvd_step also records, per workgroup, four readings of the GPU's 100 MHz
 *         wall clock (see kvd_step_timeline); the step stays asynchronous. */
int kvd_set_profiling(kvd_ctx* ctx, int32_t mode);
/* The form kvd_step takes for this context, in the terms of kvd_config.micro_batches: -1 one launch,
 * 1 a chain of kernels, n >= 2 that many groups on the library's streams. */
int kvd_step_form(const kvd_ctx* ctx);
/* Changes the form of kvd_step (same values as kvd_config.micro_batches).  Waits for the device.
 * KVD_ERR_SHAPE if the context's shapes cannot run that form. */
int kvd_set_step_form(kvd_ctx* ctx, int32_t form);
/* Pre-run calibration (Pipeline Optimization: the micro-batch size is found by a short calibration
 * before inference begins).  Runs real decode steps of `layer` — step indices first_step ..
 * first_step + steps_per_form with the queries q_steps [n_queries][B][Hq][D] (device) taken in
 * turn — in each form the context can run (chain of kernels, 2 groups, 4 groups, one launch).
 * Every form replays the same 1 untimed + steps_per_form timed steps from the same cache: the
 * layer's directory is kept on the host when the call starts and put back before each replay (its
 * slots refilled from the host store), so that all forms see the same misses — a step's time
 * follows its misses, which vary more from step to step than the forms differ.  The replays are
 * enqueued back to back and timed with HIP events on `stream`, twice per form (forms in order,
 * then in reverse order); a form's time is the smaller of its two.  The fastest form is kept and
 * reported in *chosen_form.  ms_per_step (host, 4 floats in that order, -1 for a form that cannot
 * run) may be NULL.  Afterwards the cache is where steps_per_form + 1 steps from its state at the
 * call take it; the counters of kvd_get_stats have counted every replay; `out` receives the last
 * step's output.  Synchronous.  KVD_ERR_STATE with profiling on (kvd_set_profiling), when every
 * step runs as the same chain of kernels. */
int kvd_calibrate_step_form(kvd_ctx* ctx, int32_t layer, int32_t first_step, const void* q_steps, int32_t n_queries,
                            int32_t steps_per_form, float* out, void* stream, int32_t* chosen_form,
                            float* ms_per_step);
/* Launch shape of the one-launch step.  Four numbers: how many passes of 64 pages a scoring wave
 * makes per chunk it takes (1..8); how many persistent scoring workgroups a group has (1..compute
 * units; the other compute units are left to the selection workgroups, and to attention workgroups
 * of units already selected, while scoring goes on); the attention splits per unit (at most twice
 * what kvd_create chose, at most 512 selected pages per split); and the number of groups (1..8) the
 * units of a layer are cut into: the groups follow each other through the launch, group g+1 being
 * scored while group g is selected and its missed pages are fetched, group g attended while group g+1
 * is selected — the micro-batches of SFC Disaggregation, pipelined by the order of the launch's
 * workgroups.  The context holds two shapes: multi_layer == 0 for launches of one layer (kvd_step),
 * != 0 for launches of several layers (kvd_step_layers, where consecutive layers are pipelined the
 * same way).  0 leaves a number to the library's rule.  kvd_set_step_shape waits for the device;
 * KVD_ERR_SHAPE for a shape the context cannot run.  kvd_get_step_shape writes the four numbers a
 * launch would take now (host, 4 ints).  Results do not depend on the shape. */
int kvd_set_step_shape(kvd_ctx* ctx, int32_t multi_layer, int32_t passes, int32_t scoring_workgroups, int32_t attn_splits,
                       int32_t groups);
int kvd_get_step_shape(const kvd_ctx* ctx, int32_t multi_layer, int32_t* shape);
/* Pre-run calibration of that launch shape (Pipeline Optimization: index size, cache size and
 * micro-batch size are found by a short calibration before inference begins; here the knobs are the
 * four above, which decide how scoring, selection and attention of different units overlap inside
 * the launch).  n_layers == 1 calibrates the shape of kvd_step on `layer`; n_layers > 1 that of
 * kvd_step_layers on layers [layer, layer + n_layers), with q_layers / out_layers as there.  Runs
 * the step once, so that every page the queries select is resident, then replays that same step —
 * pure GPU work — in every shape of a grid (scoring workgroups from all compute units down to a
 * quarter, 1..4 passes, splits from a quarter of the rule's to twice, 1 / 2 / 4 groups for one layer),
 * launches_per_shape timed replays each after two untimed ones, HIP events on `stream`; the eight
 * fastest and the rule's shape are timed once more, three times as long, a shape's smaller time
 * counts, and the fastest is kept if it beats the rule's shape by more than 1.5 %, else the rule's
 * (smaller differences are within what two timings of one shape differ by).  chosen_shape (host, 4 ints), us_chosen and us_rule (microseconds per layer-step in the
 * shape kept and in the rule's) may be NULL.  The replays count in kvd_get_stats; the outputs are
 * the step's.  Synchronous.  KVD_ERR_STATE if the step does not run as one launch or profiling is on. */
int kvd_calibrate_step_shape(kvd_ctx* ctx, int32_t layer, int32_t n_layers, int32_t step, const void* q_layers,
                             float* out_layers, void* stream, int32_t launches_per_shape, int32_t* chosen_shape,
                             float* us_chosen, float* us_rule);
/* Bound of every wait inside the one-launch kvd_step (micro_batches = -1), where workgroups wait on
 * counters and published words in device memory that the workgroups before them write.  Default 2 s.
 * A wait that runs out makes its workgroup leave without output and raises an error word in host
 * memory.  While the word is set kvd_get_stats and kvd_step_trace return KVD_ERR_STATE (the step that
 * failed has no valid output or trace).  The next kvd_step / kvd_step_layers call finds the word,
 * waits for the device, empties the window of every layer (the failed step may have left a
 * directory half updated), clears the word, switches the context to the chain of kernels
 * (kvd_step_form() == 1 from then on, until kvd_set_step_form says otherwise) and returns
 * KVD_ERR_STATE once, without enqueuing anything; calls after that run normally, from a cold cache.
 * kvd_cache_reset clears the word too (without changing the form).  (A limit of 0 lets tests reach
 * that path: every kernel still ends normally.) */
int kvd_set_wait_limit_us(kvd_ctx* ctx, int64_t microseconds);
/* Timeline of the last single-launch kvd_step recorded under profiling mode 2.  Synchronises the
 * device.  host_records [capacity][5] receives, for workgroup i < min(capacity, *n_workgroups) in
 * dispatch order, the clock at: start, end of its wait for its inputs (a unit's scores; the entries
 * of an attention split, which are there once its pages are resident), end of its work, exit; and
 * a tag: bits 0-7 the role (0 scoring, 1 selection + directory + fetch, 2 attention), bits 8-31
 * the unit (0 for scoring workgroups, which serve all units in turn), bits 32-63 the number of the
 * scoring workgroup or the attention split.  KVD_ERR_STATE if the step does not
 * run as one launch or none has run. */
int kvd_step_timeline(kvd_ctx* ctx, int64_t* host_records, int32_t capacity, int32_t* n_workgroups);
int kvd_get_stats(kvd_ctx* ctx, kvd_stats* host_out);   /* synchronises the device */
int kvd_reset_stats(kvd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* KVD_H */
