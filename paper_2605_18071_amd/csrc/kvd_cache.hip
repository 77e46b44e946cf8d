// Stage 2 of the decode step: the in-GPU window of recently critical pages (Attention-Based
// Cache Management; Motivation, "critical KV window") with LRU replacement, kept entirely on
// the device, and the fetch of the pages that are not resident from the pinned host store
// (Roofline section: only out-of-cache critical entries are moved).  Also the set-up kernel that
// builds the index (System Overview: mean key of each page).
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_page_copy.h"
#include "kvd_tile_layout.h"

namespace kvd {

constexpr int kResolveThreads = 256;
constexpr int kSelPerThread = KVD_MAX_TOPK / kResolveThreads;      // 8
constexpr int kBitmapWords = KVD_MAX_CAPACITY / 32;

struct ResolveArgs {
  const int32_t* capacity;   // [U] of the layer
  int32_t* resident;         // [U]
  int32_t* page_to_slot;     // [U][NP]
  int32_t* slot_page;        // [U][Cmax]
  int32_t* slot_stamp;       // [U][Cmax]
  const int32_t* sel_pages;  // [U][k]
  int32_t* sel_slots;        // [U][k]
  int32_t* hit_mask;         // [U][k]
  int32_t* evicted;          // [U][k]
  int32_t* counts;           // [U][3]
  int32_t* miss_list;        // [U][k][2]
  int32_t* miss_count;       // [U]
  unsigned long long* stats; // hits, misses, evictions
  const float* scores;       // [U][score_stride] scores of this step (lookahead eviction only)
  const int32_t* page_cluster;  // [U][NP] or null: a page's score is its cluster's (hierarchical index)
  const int32_t* seq_len;    // [B]
  int NP, Cmax, k, step, u0, lookahead, score_stride;
  int la_pool, P, Hkv;       // look-ahead pool in pages (0 = every scored page); page size and KV heads, for the valid pages of a unit
};

// One block per unit.
//  1. look every selected page up in page_to_slot; hits are re-stamped and flagged in an LDS bitmap;
//  2. e = max(0, resident + misses - capacity) pages must leave: the e smallest (stamp, page) —
//     under lookahead eviction the e smallest (score of this step, -page) — among resident slots
//     that were not hit (exact k-th smallest on the 64-bit key);
//  3. free slots and victim slots, in ascending slot order, are handed to the misses in ascending
//     page order; the directory is updated and the (page, slot) miss list written for the fetch.
__global__ __launch_bounds__(kResolveThreads) void resolve_kernel(ResolveArgs a) {
  __shared__ SelectSmem sm;
  __shared__ u32 radix_hist[kRadixBins];
  __shared__ u32 hit_bitmap[kBitmapWords];
  __shared__ int32_t assign[KVD_MAX_TOPK];
  __shared__ int n_hits, n_evicted_out;
  constexpr int NT = kResolveThreads;
  const int tid = threadIdx.x;
  const int u = blockIdx.x + a.u0;
  const int C = a.capacity[u];
  const int R = a.resident[u];
  int32_t* p2s = a.page_to_slot + (size_t)u * a.NP;
  int32_t* spage = a.slot_page + (size_t)u * a.Cmax;
  int32_t* sstamp = a.slot_stamp + (size_t)u * a.Cmax;
  const int32_t* sel = a.sel_pages + (size_t)u * a.k;
  int32_t* sslots = a.sel_slots + (size_t)u * a.k;
  int32_t* hmask = a.hit_mask + (size_t)u * a.k;
  int32_t* evout = a.evicted + (size_t)u * a.k;

  for (int i = tid; i < (C + 31) / 32; i += NT) hit_bitmap[i] = 0;
  for (int i = tid; i < a.k; i += NT) assign[i] = -1;
  if (tid == 0) { n_hits = 0; n_evicted_out = 0; }
  __syncthreads();

  // 1. lookup
  const int per = (a.k + NT - 1) / NT;               // consecutive selected entries per thread (<= 8)
  const int i0 = tid * per;
  int32_t my_page[kSelPerThread];
  int my_misses = 0, my_hits = 0;
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    my_page[j] = -2;                                 // -2: nothing here, -1..: handled below
    const int i = i0 + j;
    if (j < per && i < a.k) {
      const int p = sel[i];
      if (p < 0 || p >= a.NP) {                        // padding (or a page the caller made up)
        sslots[i] = -1;
        hmask[i] = 0;
      } else {
        const int s = p2s[p];
        if (s >= 0 && s < C) {
          sstamp[s] = a.step;
          atomicOr(&hit_bitmap[s >> 5], 1u << (s & 31));
          sslots[i] = s;
          hmask[i] = 1;
          ++my_hits;
        } else {
          my_page[j] = p;
          ++my_misses;
        }
      }
    }
  }
  if (my_hits) atomicAdd(&n_hits, my_hits);
  int m;
  int miss_rank = block_exclusive_scan<NT>(my_misses, sm.scan, m);
  const int e = (R + m - C) > 0 ? (R + m - C) : 0;

  // 2. victims
  auto page_score = [&](int p) -> float {             // this step's score of a page: its own, or its cluster's
    int at = p;
    if (a.page_cluster != nullptr) at = a.page_cluster[(size_t)u * a.NP + p];
    return at < 0 ? -INFINITY : a.scores[(size_t)u * a.score_stride + at];
  };
  auto ascending = [](float sc) -> u32 {
    const u32 x = as_u32(sc + 0.0f);
    return (x & 0x80000000u) ? ~x : (x | 0x80000000u);
  };
  // A finite look-ahead pool: the key of the pool's last member in selection order (score
  // descending, ties to the lower page) over the unit's valid pages.
  bool pooled = false;
  u64 pool_thr = ~0ull;
  if (a.lookahead && a.la_pool > 0 && e > 0) {
    int n_valid = (a.seq_len[u / a.Hkv] + a.P - 1) / a.P;
    n_valid = n_valid < a.NP ? n_valid : a.NP;
    if (a.la_pool < n_valid) {
      pooled = true;
      auto fn = [&](int p, u64& kk) -> bool {
        kk = ((u64)(~ascending(page_score(p))) << 32) | (u32)p;
        return true;
      };
      pool_thr = block_kth_smallest<NT>(fn, n_valid, a.la_pool, sm, radix_hist);
      __syncthreads();
    }
  }
  auto victim_key = [&](int s, u64& key) -> bool {
    const int p = spage[s];
    if (p < 0 || ((hit_bitmap[s >> 5] >> (s & 31)) & 1u)) return false;
    if (a.lookahead) {
      // ascending in (score, -page): the lowest score leaves first, among equals the higher page;
      // with a pool, the pages outside it before all of those, by (stamp, page)
      const float sc = page_score(p);
      const u32 asc = ascending(sc);
      if (!pooled) {
        key = ((u64)asc << 32) | (u32)(~(u32)p);
      } else if ((((u64)(~asc) << 32) | (u32)p) <= pool_thr) {
        key = (1ull << 63) | ((u64)asc << 24) | (u64)((~(u32)p) & 0xffffffu);
      } else {
        key = ((u64)((u32)sstamp[s] ^ 0x80000000u) << 24) | (u64)((u32)p & 0xffffffu);
      }
    } else {
      key = ((u64)((u32)sstamp[s] ^ 0x80000000u) << 32) | (u32)p;
    }
    return true;
  };
  u64 thr = 0;
  if (e > 0) thr = block_kth_smallest<NT>(victim_key, C, e, sm, radix_hist);

  // 3. hand out slots
  const int sper = (C + NT - 1) / NT;
  const int s0 = tid * sper;
  const int s1 = (s0 + sper) < C ? (s0 + sper) : C;
  int avail = 0;
  for (int s = s0; s < s1; ++s) {
    u64 key;
    const bool is_free = spage[s] < 0;
    const bool is_victim = e > 0 && victim_key(s, key) && key <= thr;
    avail += (is_free || is_victim) ? 1 : 0;
  }
  int total_avail;
  int rank = block_exclusive_scan<NT>(avail, sm.scan, total_avail);
  for (int s = s0; s < s1; ++s) {
    u64 key;
    const int p = spage[s];
    const bool is_free = p < 0;
    const bool is_victim = e > 0 && victim_key(s, key) && key <= thr;
    if (is_free || is_victim) {
      if (rank < m) {
        assign[rank] = s;
        if (is_victim) {
          p2s[p] = -1;
          const int at = atomicAdd(&n_evicted_out, 1);
          if (at < a.k) evout[at] = p;
        }
      }
      ++rank;
    }
  }
  __syncthreads();

  // 4. install the misses
#pragma unroll
  for (int j = 0; j < kSelPerThread; ++j) {
    const int p = my_page[j];
    if (p >= 0) {
      const int i = i0 + j;
      const int s = assign[miss_rank];
      sslots[i] = s;
      hmask[i] = 0;
      if (s >= 0) {                                    // always true while the directory is consistent
        p2s[p] = s;
        spage[s] = p;
        sstamp[s] = a.step;
      }
      a.miss_list[((size_t)u * a.k + miss_rank) * 2] = p;
      a.miss_list[((size_t)u * a.k + miss_rank) * 2 + 1] = s;
      ++miss_rank;
    }
  }
  for (int j = e + tid; j < a.k; j += NT) evout[j] = -1;
  if (tid == 0) {
    a.resident[u] = R + m - e;
    a.miss_count[u] = m;
    a.counts[u * 3 + 0] = n_hits;
    a.counts[u * 3 + 1] = m;
    a.counts[u * 3 + 2] = e;
    atomicAdd(&a.stats[0], (unsigned long long)n_hits);
    atomicAdd(&a.stats[1], (unsigned long long)m);
    atomicAdd(&a.stats[2], (unsigned long long)e);
  }
}

constexpr int kGatherThreads = 256;
constexpr int kGatherBlocksPerUnit = 8;

// Copies one page from the host store (natural layout: K[P][D] then V[P][D]) into a slot, with all
// 256 threads of the block.  TILED: the slot takes the tile layout of kvd_tile_layout.h — K moves
// in 16-byte units to permuted positions, V is transposed through LDS (`vt`, 16 x 128 elements).
template <int TILED>
__device__ __forceinline__ void copy_page(const char* __restrict__ src, char* __restrict__ dst, int P,
                                          unsigned page_bytes, uint16_t* vt) {
  const int tid = threadIdx.x;
  if (TILED == kLayoutPacked) {
    __syncthreads();                                   // previous page's readers are done with vt
    packed_copy_phase_a(src, P, dst, vt, tid);
    __syncthreads();
    packed_copy_phase_b(P, dst, vt, tid);
    return;
  }
  if (!TILED) {
    const uint4* s4 = reinterpret_cast<const uint4*>(src);
    uint4* d4 = reinterpret_cast<uint4*>(dst);
    for (unsigned o = tid; o < page_bytes / 16; o += kGatherThreads) d4[o] = s4[o];
    return;
  }
  const int tiles = P / kTileTokens;
  for (int t = 0; t < tiles; ++t) {
    char* tile = dst + (size_t)t * kTileBytes;
    __syncthreads();                                   // previous tile's readers are done with vt
    tile_copy_phase_a(src, P, t, tile, vt, tid);
    __syncthreads();
    tile_copy_phase_b(tile, vt, tid);
  }
}

// Fetch: block (x, u) copies misses x, x+8, ... of unit u from the pinned host store (read across
// the host link, 16 bytes per lane) into their slots.  With src_offset the j-th miss of the unit
// is read from store + src_offset[u][j] instead (a negative offset: nothing to copy).
template <int TILED>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(const char* __restrict__ store,   // [U][NP] pages of the layer
                                                               char* __restrict__ pool,          // [U][Cmax] slots of the layer
                                                               const int32_t* __restrict__ miss_list,
                                                               const int32_t* __restrict__ miss_count,
                                                               const int64_t* __restrict__ src_offset, int k, int NP,
                                                               int Cmax, int P, unsigned page_bytes, int u0) {
  __shared__ uint16_t vt[kTileTokens * kHeadDim];
  const int u = blockIdx.y + u0;
  const int m = miss_count[u];
  for (int j = blockIdx.x; j < m; j += gridDim.x) {
    const int page = miss_list[((size_t)u * k + j) * 2];
    const int slot = miss_list[((size_t)u * k + j) * 2 + 1];
    if (slot < 0) continue;
    const char* src;
    if (src_offset != nullptr) {
      const int64_t off = src_offset[(size_t)u * k + j];
      if (off < 0) continue;
      src = store + off;
    } else {
      src = store + ((size_t)u * NP + page) * page_bytes;
    }
    copy_page<TILED>(src, pool + ((size_t)u * Cmax + slot) * page_bytes, P, page_bytes, vt);
  }
}

// Set-up: (re)load every occupied slot of a layer from the host store, as named by slot_page.
template <int TILED>
__global__ __launch_bounds__(kGatherThreads) void refill_kernel(const char* __restrict__ store, char* __restrict__ pool,
                                                               const int32_t* __restrict__ slot_page, int NP, int Cmax,
                                                               int P, unsigned page_bytes) {
  __shared__ uint16_t vt[kTileTokens * kHeadDim];
  const int u = blockIdx.y;
  for (int s = blockIdx.x; s < Cmax; s += gridDim.x) {
    const int page = slot_page[(size_t)u * Cmax + s];
    if (page < 0) continue;
    copy_page<TILED>(store + ((size_t)u * NP + page) * page_bytes, pool + ((size_t)u * Cmax + s) * page_bytes, P,
                     page_bytes, vt);
  }
}

// Index build: one block per page, one thread per dimension; the sum runs over the page's valid
// tokens in token order in fp64 and is rounded once to the KV dtype.
template <bool BF16>
__global__ __launch_bounds__(kHeadDim) void summaries_kernel(const uint16_t* __restrict__ store,   // [U][NP][2][P][D]
                                                            uint16_t* __restrict__ summ,          // [U][NP][D]
                                                            const int32_t* __restrict__ seq_len, int NP, int P,
                                                            int Hkv) {
  const int page = blockIdx.x, u = blockIdx.y, d = threadIdx.x;
  const int b = u / Hkv;
  int n = seq_len[b] - page * P;
  n = n < P ? n : P;
  uint16_t* out = summ + ((size_t)u * NP + page) * kHeadDim + d;
  if (n <= 0) { *out = 0; return; }
  const uint16_t* kp = store + ((size_t)u * NP + page) * (size_t)(2 * P * kHeadDim) + d;
  double acc = 0.0;
  for (int t0 = 0; t0 < n; t0 += 16) {
    uint16_t raw[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int t = (t0 + j) < n ? (t0 + j) : (n - 1);
      raw[j] = kp[(size_t)t * kHeadDim];
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (t0 + j < n) {
        float f;
        if (BF16) {
          f = as_f32((u32)raw[j] << 16);
        } else {
          f = (float)__builtin_bit_cast(_Float16, raw[j]);
        }
        acc += (double)f;
      }
    }
  }
  *out = f64_to_kv<BF16>(acc / (double)n);
}

// Decoding appends the key and value of the token just generated to the KV store (Background,
// "KV Cache Basics").  One block per unit: the token lands at position seq_len[b] of the host
// store (written across the host link), in the slot of its page if that page is resident, and the
// page's index entry is recomputed as the mean over its valid tokens including the new one (fp64,
// token order, rounded once — the same definition as summaries_kernel).
template <bool BF16, int TILED>
__global__ __launch_bounds__(256) void append_kernel(uint16_t* __restrict__ store,          // [U][NP][2][P][D] of the layer
                                                    uint16_t* __restrict__ summ,           // [U][NP][D]
                                                    char* __restrict__ pool,               // [U][Cmax] slots
                                                    const int32_t* __restrict__ slot_page, // [U][Cmax]
                                                    const int32_t* __restrict__ capacity,  // [U]
                                                    const uint16_t* __restrict__ k_new,    // [U][D]
                                                    const uint16_t* __restrict__ v_new,    // [U][D]
                                                    const int32_t* __restrict__ seq_len, int NP, int P, int Cmax,
                                                    int Hkv, unsigned page_bytes) {
  __shared__ int found_slot;
  const int u = blockIdx.x, tid = threadIdx.x;
  const int b = u / Hkv;
  const int t = seq_len[b];
  const int page = t / P, o = t % P;
  if (page >= NP) return;                                // no room: the host checks this before launching
  if (tid == 0) found_slot = -1;
  __syncthreads();
  uint16_t* kpage = store + ((size_t)u * NP + page) * (size_t)(2 * P * kHeadDim);
  uint16_t* vpage = kpage + (size_t)P * kHeadDim;
  const uint16_t* kn = k_new + (size_t)u * kHeadDim;
  const uint16_t* vn = v_new + (size_t)u * kHeadDim;

  // 1. the host store: 16 lanes x 16 bytes for K, 16 for V
  if (tid < 32) {
    const int ch = tid & 15;
    const uint4 val = *reinterpret_cast<const uint4*>((tid < 16 ? kn : vn) + ch * 8);
    *reinterpret_cast<uint4*>((tid < 16 ? kpage : vpage) + (size_t)o * kHeadDim + ch * 8) = val;
  }

  // 2. is the page resident?
  const int C = capacity[u];
  for (int s = tid; s < C; s += 256)
    if (slot_page[(size_t)u * Cmax + s] == page) found_slot = s;      // at most one slot holds the page
  __syncthreads();
  const int slot = found_slot;
  if (slot >= 0 && tid < kHeadDim) {
    char* sl = pool + ((size_t)u * Cmax + slot) * page_bytes;
    const int d = tid;
    if (TILED == kLayoutPacked) {
      // packed layout (kvd_tile_layout.h): K element [o][d] in unit (c, g, o), V element [o][d] in
      // unit (c, o / 4, d % 16) at element 4 ((d % 32) / 16) + o % 4
      const int c = d >> 5, r32 = d & 31;
      uint16_t* kdst = reinterpret_cast<uint16_t*>(sl + (size_t)((c * 4 + (r32 >> 3)) * P + o) * 16) + (d & 7);
      uint16_t* vdst = reinterpret_cast<uint16_t*>(sl + (size_t)P * kRowBytes + (size_t)((c * (P >> 2) + (o >> 2)) * 16 + (d & 15)) * 16) +
                       4 * (r32 >> 4) + (o & 3);
      *kdst = kn[d];
      *vdst = vn[d];
    } else if (TILED) {
      // tile layout (kvd_tile_layout.h): K element [row][d] sits in chunk d/32, lane row + 16 ((d%32)/8),
      // element d%8; V element [row][d] in chunk d/32, lane d%16 + 16 (row/4), element 4 ((d%32)/16) + row%4
      char* tile = sl + (size_t)(o / kTileTokens) * kTileBytes;
      const int row = o % kTileTokens;
      const int c = d >> 5, r32 = d & 31;
      uint16_t* kdst = reinterpret_cast<uint16_t*>(tile + (c * 64 + (r32 >> 3) * 16 + row) * 16) + (d & 7);
      uint16_t* vdst = reinterpret_cast<uint16_t*>(tile + kTilePartBytes + (c * 64 + (row >> 2) * 16 + (d & 15)) * 16) +
                       4 * (r32 >> 4) + (row & 3);
      *kdst = kn[d];
      *vdst = vn[d];
    } else {
      uint16_t* k16 = reinterpret_cast<uint16_t*>(sl);
      k16[(size_t)o * kHeadDim + d] = kn[d];
      k16[(size_t)(P + o) * kHeadDim + d] = vn[d];
    }
  }

  // 3. the index entry of the page: tokens 0..o-1 from the host store, then the new key
  if (tid < kHeadDim) {
    const int d = tid;
    double acc = 0.0;
    for (int t0 = 0; t0 < o; t0 += 16) {
      uint16_t raw[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int tt = (t0 + j) < o ? (t0 + j) : (o - 1);
        raw[j] = kpage[(size_t)tt * kHeadDim + d];
      }
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (t0 + j < o) acc += (double)(BF16 ? as_f32((u32)raw[j] << 16) : (float)__builtin_bit_cast(_Float16, raw[j]));
    }
    const uint16_t kb = kn[d];
    acc += (double)(BF16 ? as_f32((u32)kb << 16) : (float)__builtin_bit_cast(_Float16, kb));
    summ[((size_t)u * NP + page) * kHeadDim + d] = f64_to_kv<BF16>(acc / (double)(o + 1));
  }
}

__global__ void advance_kernel(int32_t* seq_len, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) seq_len[b] += 1;
}

__global__ void fill_i32_kernel(int32_t* p, int32_t v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

}  // namespace kvd

hipError_t kvd_launch_resolve(kvd_ctx* c, int layer, int step, const int32_t* sel_pages, int32_t* sel_slots,
                              int32_t* hit_mask, int32_t* evicted, int32_t* counts, int u0, int u1, hipStream_t s) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  if (c->d_page_to_slot == nullptr) return hipErrorInvalidValue;   // (contexts of the register-resident path have no such table)
  ResolveArgs a;
  const size_t lu = (size_t)layer * c->U;
  a.capacity = c->d_capacity + lu;
  a.resident = c->d_resident + lu;
  a.page_to_slot = c->d_page_to_slot + lu * c->NP;
  a.slot_page = c->d_slot_page + lu * c->Cmax;
  a.slot_stamp = c->d_slot_stamp + lu * c->Cmax;
  a.sel_pages = sel_pages;
  a.sel_slots = sel_slots;
  a.hit_mask = hit_mask;
  a.evicted = evicted;
  a.counts = counts;
  a.miss_list = c->d_miss_list;
  a.miss_count = c->d_miss_count;
  a.stats = c->d_stats;
  a.NP = c->NP; a.Cmax = c->Cmax; a.k = c->k; a.step = step; a.u0 = u0;
  a.lookahead = c->cfg.policy == KVD_EVICT_LOOKAHEAD ? 1 : 0;
  a.la_pool = c->cfg.lookahead_pool; a.P = c->P; a.Hkv = c->Hkv;
  a.seq_len = c->d_seq_len;
  a.scores = c->last_scores;
  a.page_cluster = c->Nc > 0 ? c->d_page_cluster + lu * c->NP : nullptr;
  a.score_stride = c->Nc > 0 ? c->Nc : c->NP;
  hipLaunchKernelGGL(resolve_kernel, dim3(u1 - u0), dim3(kResolveThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t kvd_launch_gather(kvd_ctx* c, int layer, int u0, int u1, hipStream_t s, const char* src_base,
                             const int64_t* src_offset) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  const int lp = layer % c->Lp;
  const char* store = src_offset ? src_base : c->store_dev + (size_t)lp * c->U * c->NP * c->page_bytes;
  char* pool = c->pool + (size_t)layer * c->U * c->Cmax * c->page_bytes;
#define KVD_GATHER(LAYOUT)                                                                                              \
  hipLaunchKernelGGL(gather_kernel<LAYOUT>, dim3(kGatherBlocksPerUnit, u1 - u0), dim3(kGatherThreads), 0, s, store, pool, \
                     c->d_miss_list, c->d_miss_count, src_offset, c->k, c->NP, c->Cmax, c->P, (unsigned)c->page_bytes, u0)
  if (c->tiled == kLayoutPacked) KVD_GATHER(kLayoutPacked);
  else if (c->tiled) KVD_GATHER(kLayoutTiles);
  else KVD_GATHER(kLayoutNatural);
#undef KVD_GATHER
  return hipGetLastError();
}

hipError_t kvd_launch_refill(kvd_ctx* c, int layer, hipStream_t s) {
  using namespace kvd;
  const int lp = layer % c->Lp;
  const char* store = c->store_dev + (size_t)lp * c->U * c->NP * c->page_bytes;
  char* pool = c->pool + (size_t)layer * c->U * c->Cmax * c->page_bytes;
  const int32_t* slot_page = c->d_slot_page + (size_t)layer * c->U * c->Cmax;
  const int bx = c->Cmax < 64 ? c->Cmax : 64;
#define KVD_REFILL(LAYOUT)                                                                                          \
  hipLaunchKernelGGL(refill_kernel<LAYOUT>, dim3(bx, c->U), dim3(kGatherThreads), 0, s, store, pool, slot_page, c->NP, \
                     c->Cmax, c->P, (unsigned)c->page_bytes)
  if (c->tiled == kLayoutPacked) KVD_REFILL(kLayoutPacked);
  else if (c->tiled) KVD_REFILL(kLayoutTiles);
  else KVD_REFILL(kLayoutNatural);
#undef KVD_REFILL
  return hipGetLastError();
}

hipError_t kvd_launch_build_summaries(kvd_ctx* c, int layer, hipStream_t s) {
  using namespace kvd;
  const int lp = layer % c->Lp;
  const uint16_t* store = reinterpret_cast<const uint16_t*>(c->store_dev + (size_t)lp * c->U * c->NP * c->page_bytes);
  uint16_t* summ = reinterpret_cast<uint16_t*>(c->summaries) + (size_t)layer * c->U * c->NP * kHeadDim;
  dim3 grid(c->NP, c->U);
  if (c->bf16)
    hipLaunchKernelGGL(summaries_kernel<true>, grid, dim3(kHeadDim), 0, s, store, summ, c->d_seq_len, c->NP, c->P, c->Hkv);
  else
    hipLaunchKernelGGL(summaries_kernel<false>, grid, dim3(kHeadDim), 0, s, store, summ, c->d_seq_len, c->NP, c->P, c->Hkv);
  return hipGetLastError();
}

hipError_t kvd_launch_append(kvd_ctx* c, int layer, const void* k_new, const void* v_new, hipStream_t s) {
  using namespace kvd;
  const size_t lu = (size_t)layer * c->U;
  uint16_t* store = reinterpret_cast<uint16_t*>(const_cast<char*>(c->store_dev) + (size_t)layer * c->U * c->NP * c->page_bytes);
  uint16_t* summ = reinterpret_cast<uint16_t*>(c->summaries) + lu * c->NP * kHeadDim;
  char* pool = c->pool + lu * c->Cmax * c->page_bytes;
  const int32_t* slot_page = c->d_slot_page + lu * c->Cmax;
  const int32_t* cap = c->d_capacity + lu;
  const uint16_t* kn = reinterpret_cast<const uint16_t*>(k_new);
  const uint16_t* vn = reinterpret_cast<const uint16_t*>(v_new);
  dim3 grid(c->U), block(256);
#define KVD_APPEND(BF, TL)                                                                                          \
  hipLaunchKernelGGL((append_kernel<BF, TL>), grid, block, 0, s, store, summ, pool, slot_page, cap, kn, vn, c->d_seq_len, \
                     c->NP, c->P, c->Cmax, c->Hkv, (unsigned)c->page_bytes)
  if (c->bf16) {
    if (c->tiled == kLayoutPacked) KVD_APPEND(true, kLayoutPacked); else if (c->tiled) KVD_APPEND(true, kLayoutTiles); else KVD_APPEND(true, kLayoutNatural);
  } else {
    if (c->tiled == kLayoutPacked) KVD_APPEND(false, kLayoutPacked); else if (c->tiled) KVD_APPEND(false, kLayoutTiles); else KVD_APPEND(false, kLayoutNatural);
  }
#undef KVD_APPEND
  return hipGetLastError();
}

hipError_t kvd_launch_advance(kvd_ctx* c, hipStream_t s) {
  hipLaunchKernelGGL(kvd::advance_kernel, dim3((c->B + 63) / 64), dim3(64), 0, s, c->d_seq_len, c->B);
  return hipGetLastError();
}

hipError_t kvd_launch_fill_i32(int32_t* p, int32_t v, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(kvd::fill_i32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, v, n);
  return hipGetLastError();
}
