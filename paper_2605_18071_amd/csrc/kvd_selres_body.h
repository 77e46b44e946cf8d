// Selection, cache-directory update and fetch for one unit by one workgroup of NT threads:
// exact Top-K selection of the scored pages (Background: "retrieving only the Top-K"), the
// directory update for the same unit (Attention-Based Cache Management with LRU replacement),
// and the fetch of the unit's missed pages from the pinned host store (only out-of-cache entries
// move — Roofline section).  Shared by the stand-alone kernel and the single-launch layer-step
// kernel.
//
// Selection and victim choice are both "the n smallest of distinct 64-bit keys" problems and share
// one two-level routine: an LDS histogram over a monotone bucket function narrows the answer to
// one bucket, whose few members are ranked exactly.  The items stay in registers; only a bucket
// with more than 1024 members (degenerate inputs, e.g. all scores equal) falls back to radix
// refinement.  The page -> slot map of the unit is rebuilt in LDS from the slot array at every
// launch, so a lookup never waits on a dependent global load; every global load the block needs
// is issued in its first instructions.
#pragma once
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_page_copy.h"

namespace kvd {

constexpr int kListCap = 1024;
constexpr uint16_t kAbsent = 0xffffu;

struct FastArgs {
  const float* scores;        // [U][NP]
  const int32_t* seq_len;     // [B]
  int32_t* sel_pages;         // [U][k]: written by the selection, read when only resolving
  const int32_t* capacity;    // [U] of the layer
  int32_t* resident;          // [U]
  int32_t* slot_page;         // [U][Cmax]
  int32_t* slot_stamp;        // [U][Cmax]
  int32_t* sel_slots;         // [U][k]
  u64* sel_entry;             // [U][k] or null: (valid, slot, page) entries for the attention workgroups of the same launch; zero between launches
  int32_t* hit_mask;          // [U][k]
  int32_t* evicted;           // [U][k]
  int32_t* counts;            // [U][3]
  int32_t* miss_list;         // [U][k][2]
  int32_t* miss_count;        // [U]
  unsigned long long* stats;  // hits, misses, evictions
  const char* store;          // host store of the layer, [U][NP] pages (device-visible address)
  char* pool;                 // slot pool of the layer, [U][Cmax] slots
  int NP, P, k, Cmax, sink, recent, Hkv, step, u0, do_gather, tiled;
  int lookahead;              // victims by lowest current-step score (needs `scores`) instead of by age
  int la_pool;                // look-ahead pool in pages (0 = every scored page): resident pages outside the step's la_pool
                              // best-scoring pages leave first, least recently selected first
  const int32_t* page_cluster;  // [U][NP] or null: the victims' scores are those of the pages' clusters
  int score_stride;           // scores of unit u start at scores + u * score_stride (NP, or the number of centroids)
  unsigned page_bytes;
};

// What the attention workgroups of the same launch read instead of sel_pages / sel_slots: one
// 64-bit word per selected entry, bit 63 = published, bits 32..47 the slot (0xffff = none), the
// low word the page (-1 = padding).  A word is published once the page's bytes are in its slot.
__device__ __forceinline__ u64 pack_sel_entry(int page, int slot) {
  return (1ull << 63) | ((u64)((u32)slot & 0xffffu) << 32) | (u64)(u32)page;
}

// This step's score of a resident page as lookahead eviction sees it: the page's own score, or with
// the hierarchical index the score of its cluster (-inf for a page of no cluster: it leaves first).
template <bool HANDOFF>
__device__ __forceinline__ float victim_score(const FastArgs& a, int u, int page) {
  int at = page;
  if (a.page_cluster != nullptr) {
    at = a.page_cluster[(size_t)u * a.NP + page];
    if (at < 0) return -INFINITY;
  }
  const float* sc = a.scores + (size_t)u * a.score_stride + at;
  return HANDOFF ? load_agent(sc) : *sc;
}

template <int NT>
struct FastSmem {
  static constexpr int NW = NT / kWave;
  static constexpr int kCopyGroups = NT / 256;           // tiles copied at a time
  union {
    struct {
      u32 hist[kRadixBins];
      u64 cand[kListCap];
    } sel;
    uint16_t vt[kCopyGroups][kTileTokens * kHeadDim];    // V tiles in flight during the fetch
  } a;
  uint16_t p2s[KVD_FAST_MAX_PAGES];                      // page -> slot of this unit, kAbsent = not resident
  uint16_t sel[KVD_MAX_TOPK];                            // selected pages (kAbsent = padding)
  uint16_t assign[KVD_MAX_TOPK];                         // slot handed to the i-th miss
  u32 hit_bitmap[KVD_FAST_MAX_CAPACITY / 32];
  int scan[2][NW];
  float red_min[NW], red_max[NW];
  int red_cnt[NW];
  u64 thr;
  int cand_n, bin, below, n_ev;
  SelectSmem generic;
};

__device__ __forceinline__ u32 fast_descending_key(float s) {
  const u32 x = as_u32(s + 0.0f);                    // -0 -> +0 so that the two zeros tie
  const u32 asc = (x & 0x80000000u) ? ~x : (x | 0x80000000u);
  return ~asc;
}
// Key of the selection order (best page first); it also decides membership of the look-ahead pool.
__device__ __forceinline__ u64 selection_order_key(float s, int page) {
  return ((u64)fast_descending_key(s) << 32) | (u32)page;
}

// Exclusive prefix sum over the block with one barrier: the wave totals alternate between two
// LDS rows (`flip` is the caller's per-thread call counter), so a call never overwrites totals
// that slower waves may still be reading from the call before.
template <int NT>
__device__ __forceinline__ int fast_scan(int v, FastSmem<NT>& sm, int& flip, int& total) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int inc = wave_inclusive_scan(v);
  int* row = sm.scan[flip & 1];
  ++flip;
  if (lane == kWave - 1) row[w] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const int t = row[i];
    base += i < w ? t : 0;
    tot += t;
  }
  total = tot;
  return base + inc - v;
}

// Items j = 0..IPT-1 of every thread: bkt(j) in [0, 2047], or -1 for "not a candidate"; key(j)
// distinct; key1 < key2 implies bkt1 <= bkt2.  sm.a.sel.hist must be zero and sm.cand_n zero on
// entry (with a barrier since).  Returns the need-th smallest key among the candidates
// (1 <= need <= number of candidates).  `refine(bin, r)` is called by all threads when the
// decisive bucket holds more than kListCap items and must return the r-th smallest key of that
// bucket.  Ends with the block synchronised.
template <int NT, int IPT, class KeyOf, class BktOf, class Refine>
__device__ __forceinline__ u64 two_level_select(KeyOf key, BktOf bkt, int need, FastSmem<NT>& sm, int& flip,
                                                Refine refine) {
  const int tid = threadIdx.x;
  u32* hist = sm.a.sel.hist;
#pragma unroll
  for (int j = 0; j < IPT; ++j) {
    const int bj = bkt(j);
    if (bj >= 0) atomicAdd(&hist[bj], 1u);
  }
  __syncthreads();
  constexpr int BPT = kRadixBins / NT;
  int local = 0;
#pragma unroll
  for (int j = 0; j < BPT; ++j) local += (int)hist[tid * BPT + j];
  int total;
  int ex = fast_scan<NT>(local, sm, flip, total);
  if (ex < need && need <= ex + local) {             // exactly one thread
    int b = tid * BPT;
    for (int j = 0; j < BPT; ++j, ++b) {
      const int c = (int)hist[b];
      if (need <= ex + c) break;
      ex += c;
    }
    sm.bin = b;
    sm.below = ex;
  }
  __syncthreads();
  const int bin = sm.bin;
  const int r = need - sm.below;
  const int m = (int)hist[bin];
  if (m > kListCap) return refine(bin, r);
#pragma unroll
  for (int j = 0; j < IPT; ++j)
    if (bkt(j) == bin) sm.a.sel.cand[atomicAdd(&sm.cand_n, 1)] = key(j);
  __syncthreads();
  for (int c = tid; c < m; c += NT) {
    const u64 mine = sm.a.sel.cand[c];
    int rank = 0;
    for (int x = 0; x < m; ++x) rank += sm.a.sel.cand[x] < mine ? 1 : 0;
    if (rank == r - 1) sm.thr = mine;
  }
  __syncthreads();
  return sm.thr;
}

// Victim key of lookahead eviction: ascending in (score, -page), so that the lowest score leaves
// first and, among equal scores, the higher page.
__device__ __forceinline__ u64 lookahead_victim_key(float s, int page) {
  const u32 x = as_u32(s + 0.0f);
  const u32 asc = (x & 0x80000000u) ? ~x : (x | 0x80000000u);
  return ((u64)asc << 32) | (u32)(~(u32)page);
}

// With a finite look-ahead pool the victim order is: pages outside the pool by (stamp, page), then
// pool pages by (score, -page).  One 64-bit key carries both (pages are below 2^24): bit 63 = in
// the pool, then the 32-bit stamp or score key, then the page or its complement.
__device__ __forceinline__ u64 pooled_victim_key(bool in_pool, float s, int stamp, int page) {
  if (!in_pool) return ((u64)((u32)stamp ^ 0x80000000u) << 24) | (u64)((u32)page & 0xffffffu);
  const u32 x = as_u32(s + 0.0f);
  const u32 asc = (x & 0x80000000u) ? ~x : (x | 0x80000000u);
  return (1ull << 63) | ((u64)asc << 24) | (u64)((~(u32)page) & 0xffffffu);
}
__device__ __forceinline__ int victim_bucket(long long age, int page, int NP) {
  // one group of 32 buckets per age (step - stamp) below 64, split by page range; everything older
  // shares bucket 0; the newest class (age <= 1) shares bucket 2047
  if (age >= 64) return 0;
  if (age <= 1) return 2047;
  return (int)(2048 - 32 * age) + (int)(((long long)page * 32) / NP);
}

// All NT threads of a workgroup, for unit u.  DO_SELECT: scores -> sel_pages (Top-K, ties to the
// lower page, sink/recent pages forced, ascending page order, -1 padding).  DO_RESOLVE: sel_pages
// -> directory update, slots, hit mask, evicted list, counts, the (page, slot) miss list and,
// with do_gather, the copy of the missed pages into their slots.  HANDOFF: the scores were
// written by other workgroups of the same launch and are read with device-scope loads, and the
// selection is handed to the launch's attention workgroups through a.sel_entry: an entry that hits
// is published at once, an entry that missed when the fetched pages have been written through.
// Needs NP <= NT * IPT, Cmax <= KVD_FAST_MAX_CAPACITY, k <= KVD_MAX_TOPK.
// scores_ready() (HANDOFF only) is called by all threads once everything that does not depend on
// the scores has been done; it waits for them and returns false to give up.  Returns false then.
// SEL_IN_LDS (with HANDOFF and without DO_SELECT): scores_ready() itself produces the selection —
// the hierarchical index's cluster selection, by the same workgroup — and leaves it in sm.sel
// (16-bit pages, kAbsent = padding) and in a.sel_pages; nothing is read back from global memory.
struct ScoresAlreadyThere { __device__ bool operator()() const { return true; } };
template <int NT, int IPT, bool DO_SELECT, bool DO_RESOLVE, bool HANDOFF, class ScoresReady = ScoresAlreadyThere,
          bool SEL_IN_LDS = false>
__device__ __forceinline__ bool select_resolve_body(const FastArgs& a, int u, FastSmem<NT>& sm,
                                                    ScoresReady scores_ready = ScoresReady()) {
  constexpr int CPT = KVD_FAST_MAX_CAPACITY / NT;
  constexpr int KPT = KVD_MAX_TOPK / NT;
  constexpr int NW = NT / kWave;
  constexpr int kCopyGroups = FastSmem<NT>::kCopyGroups;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int b = u / a.Hkv;
  const int k = a.k;
  int flip = 0;

  // ---- every global load of the block, issued up front
  int32_t* spage = a.slot_page + (size_t)u * a.Cmax;
  int32_t* sstamp = a.slot_stamp + (size_t)u * a.Cmax;
  int sp[CPT], ss[CPT];                               // page in slot (-1 free, -2 no such slot), stamp
  int C = 0, R = 0;
  if (DO_RESOLVE) {
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const int s = tid * CPT + j;
      sp[j] = s < a.Cmax ? spage[s] : -2;
      ss[j] = s < a.Cmax ? sstamp[s] : 0;
    }
    C = a.capacity[u];
    R = a.resident[u];
  }
  // Page ownership: a wave owns 64 * IPT consecutive pages; its q-th 16-byte load covers 256 of
  // them (1 KiB contiguous), lane l taking four.  Item j of a lane is page_of(j).
  static_assert(IPT % 4 == 0, "four consecutive pages per load");
  const int wave_p0 = w * (kWave * IPT);
  auto page_of = [&](int j) -> int { return wave_p0 + (j >> 2) * (4 * kWave) + 4 * lane + (j & 3); };
  float s[IPT];
  int seq = 0;
  auto load_scores = [&]() {
    const float* sc = a.scores + (size_t)u * a.NP;
    if ((a.NP & 3) == 0) {
      // bounds-checked by the buffer descriptor: pages beyond NP read as 0 and are never valid
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(sc), 0, a.NP * 4, 0x00020000);
#pragma unroll
      for (int q4 = 0; q4 < IPT / 4; ++q4) {
        const int off = page_of(4 * q4) * 4;
        // HANDOFF: device-scope load (the scores come from other workgroups of this launch)
        const u32x4_t v = HANDOFF ? __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 16)
                                  : __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
        s[4 * q4] = as_f32(v.x); s[4 * q4 + 1] = as_f32(v.y); s[4 * q4 + 2] = as_f32(v.z); s[4 * q4 + 3] = as_f32(v.w);
      }
    } else {
#pragma unroll
      for (int j = 0; j < IPT; ++j) {
        const int p = page_of(j);
        s[j] = p < a.NP ? (HANDOFF ? load_agent(sc + p) : sc[p]) : 0.f;
      }
    }
  };
  if (DO_SELECT) {
    if (!HANDOFF) load_scores();                       // (with HANDOFF the scores may not be complete yet)
    seq = a.seq_len[b];
  } else if (!SEL_IN_LDS) {
    for (int i = tid; i < k; i += NT) {
      const int p = a.sel_pages[(size_t)u * k + i];
      sm.sel[i] = (p >= 0 && p < a.NP) ? (uint16_t)p : kAbsent;
    }
  }

  // ---- LDS set-up while the loads are in flight
  for (int i = tid; i < kRadixBins; i += NT) sm.a.sel.hist[i] = 0;
  if (DO_RESOLVE) {
    u32* p2s32 = reinterpret_cast<u32*>(sm.p2s);
    for (int i = tid; i < (a.NP + 1) / 2; i += NT) p2s32[i] = 0xffffffffu;
    for (int i = tid; i < KVD_FAST_MAX_CAPACITY / 32; i += NT) sm.hit_bitmap[i] = 0;
    for (int i = tid; i < k; i += NT) sm.assign[i] = kAbsent;
  }
  if (tid == 0) { sm.cand_n = 0; sm.n_ev = 0; }
  __syncthreads();
  float vs[CPT];                                       // lookahead eviction: this step's score of the page in each slot
  if (DO_RESOLVE) {
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const int sl = tid * CPT + j;
      if (sl >= C && sp[j] != -2) sp[j] = -2;          // slots beyond this unit's capacity do not exist
      if (sp[j] >= 0) sm.p2s[sp[j]] = (uint16_t)sl;
    }
  }
  if (HANDOFF) {
    // everything that does not need the scores is done: now wait for them
    if (!scores_ready()) return false;
    if (DO_SELECT) load_scores();
  }
  if (DO_RESOLVE) {
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      vs[j] = 0.f;
      if (a.lookahead && sp[j] >= 0) vs[j] = victim_score<HANDOFF>(a, u, sp[j]);
    }
  }

  // ---- selection
  if (DO_SELECT) {
    int n_valid = (seq + a.P - 1) / a.P;
    n_valid = n_valid < a.NP ? n_valid : a.NP;
    const int k_eff = k < n_valid ? k : n_valid;
    const int recent_from = n_valid - a.recent;
    // Which of this lane's pages are free to compete and which are forced, four consecutive pages
    // at a time: free = [sink, recent_from), forced = the other valid pages.
    u32 free_mask = 0, forced_mask = 0;               // bit j: page_of(j)
#pragma unroll
    for (int q4 = 0; q4 < IPT / 4; ++q4) {
      const int base = page_of(4 * q4);
      auto upto = [&](int bound) -> u32 {              // bits of the group's pages below `bound`
        const int n = bound - base;
        return (1u << (n < 0 ? 0 : (n > 4 ? 4 : n))) - 1u;
      };
      const u32 fr = upto(recent_from) & ~upto(a.sink);
      free_mask |= fr << (4 * q4);
      forced_mask |= (upto(n_valid) & ~fr) << (4 * q4);
    }
    float fmin = INFINITY, fmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const bool fr = (free_mask >> j) & 1u;
      fmin = fminf(fmin, fr ? s[j] : INFINITY);
      fmax = fmaxf(fmax, fr ? s[j] : -INFINITY);
    }
    int n_forced = __popc(forced_mask);
    fmin = wave_allreduce_min(fmin);
    fmax = wave_allreduce_max(fmax);
    n_forced = wave_inclusive_scan(n_forced);          // lane 63 holds the wave's count
    n_forced = __builtin_amdgcn_readlane(n_forced, 63);
    if (lane == 0) { sm.red_min[w] = fmin; sm.red_max[w] = fmax; sm.red_cnt[w] = n_forced; }
    __syncthreads();
    fmin = sm.red_min[0]; fmax = sm.red_max[0]; n_forced = sm.red_cnt[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) {
      fmin = fminf(fmin, sm.red_min[i]);
      fmax = fmaxf(fmax, sm.red_max[i]);
      n_forced += sm.red_cnt[i];
    }
    const int k_free = k_eff - n_forced;
    const float range = fmax - fmin;
    const float inv = range > 0.f ? 2047.0f / range : 0.f;
    auto bucket_of = [&](float v) -> int { return (int)fminf(fmaxf((fmax - v) * inv, 0.f), 2047.f); };
    // every free page's bucket, computed once and kept (two per register); 0xffff = not free
    u32 bk2[IPT / 2];
#pragma unroll
    for (int j = 0; j < IPT; j += 2) {
      const u32 b0 = ((free_mask >> j) & 1u) ? (u32)bucket_of(s[j]) : 0xffffu;
      const u32 b1 = ((free_mask >> (j + 1)) & 1u) ? (u32)bucket_of(s[j + 1]) : 0xffffu;
      bk2[j / 2] = b0 | (b1 << 16);
    }
    auto bucket_at = [&](int j) -> int { return (int)((bk2[j >> 1] >> (16 * (j & 1))) & 0xffffu); };
    auto key_of = [&](int j) -> u64 { return ((u64)fast_descending_key(s[j]) << 32) | (u32)page_of(j); };
    auto bkt_of = [&](int j) -> int { const int bb = bucket_at(j); return bb == 0xffff ? -1 : bb; };
    u64 thr = 0;
    if (k_free > 0) {
      const float* sc = a.scores + (size_t)u * a.NP;
      auto refine = [&](int bin, int r) -> u64 {
        auto fn = [&](int i, u64& kk) -> bool {
          if (i < a.sink || i >= recent_from) return false;
          const float v = HANDOFF ? load_agent(sc + i) : sc[i];
          if (bucket_of(v) != bin) return false;
          kk = ((u64)fast_descending_key(v) << 32) | (u32)i;
          return true;
        };
        return block_kth_smallest<NT>(fn, n_valid, r, sm.generic, sm.a.sel.hist);
      };
      thr = two_level_select<NT, IPT>(key_of, bkt_of, k_free, sm, flip, refine);
    }
    // a page in a bucket before the decisive one is in, one in a later bucket is out; only the
    // members of the decisive bucket are compared with the threshold key
    const int bin = k_free > 0 ? sm.bin : -1;
    u32 take = forced_mask;                            // bit j: page_of(j) is selected
#pragma unroll
    for (int j = 0; j < IPT; ++j) {
      const int bb = bucket_at(j);
      bool t = bb < bin;
      if (bb == bin) t = key_of(j) <= thr;
      take |= t ? (1u << j) : 0u;
    }
    int cnt4[IPT / 4];
    int cnt = __popc(take);
#pragma unroll
    for (int q4 = 0; q4 < IPT / 4; ++q4) cnt4[q4] = __popc((take >> (4 * q4)) & 15u);
    // output in ascending page order = (wave, load, lane, element): one block scan over the
    // lanes' totals gives the wave's first position, wave scans per load give the rest
    int total;
    const int lane_pos = fast_scan<NT>(cnt, sm, flip, total);
    int pos_q = __builtin_amdgcn_readfirstlane(lane_pos);   // lane 0: what the waves before this one selected
    int32_t* out = a.sel_pages + (size_t)u * k;
#pragma unroll
    for (int q4 = 0; q4 < IPT / 4; ++q4) {
      const int inc = wave_inclusive_scan(cnt4[q4]);
      int pos = pos_q + inc - cnt4[q4];
      pos_q += __builtin_amdgcn_readlane(inc, kWave - 1);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = 4 * q4 + e;
        if ((take >> j) & 1u) {
          if (pos < k) {
            const int p = page_of(j);
            sm.sel[pos] = (uint16_t)p;
            out[pos] = p;
          }
          ++pos;
        }
      }
    }
    for (int i = k_eff + tid; i < k; i += NT) {
      sm.sel[i] = kAbsent;
      out[i] = -1;
    }
    if (!DO_RESOLVE) return true;
    // the histogram and the candidate counter serve the victim choice next
    for (int i = tid; i < kRadixBins; i += NT) sm.a.sel.hist[i] = 0;
    if (tid == 0) sm.cand_n = 0;
  }
  __syncthreads();

  // ---- resolve: lookup in the LDS map
  int32_t* sslots = a.sel_slots + (size_t)u * k;
  int32_t* hmask = a.hit_mask + (size_t)u * k;
  int32_t* evout = a.evicted + (size_t)u * k;
  u64* entry = HANDOFF ? a.sel_entry + (size_t)u * k : nullptr;
  const int per = (k + NT - 1) / NT;                  // consecutive selected entries per thread
  const int i0 = tid * per;
  int my_page[KPT], my_slot[KPT];                     // this thread's misses and the slots they get
  int my_misses = 0, my_hits = 0;
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    my_page[j] = -2;
    my_slot[j] = -1;
    const int i = i0 + j;
    if (j < per && i < k) {
      const int p = sm.sel[i];
      if (p == kAbsent) {                             // padding (or a page the caller made up)
        sslots[i] = -1;
        if (HANDOFF) store_agent(entry + i, pack_sel_entry(-1, -1));
        hmask[i] = 0;
      } else {
        const int sl = sm.p2s[p];
        if (sl != kAbsent) {
          sstamp[sl] = a.step;
          atomicOr(&sm.hit_bitmap[sl >> 5], 1u << (sl & 31));
          sslots[i] = sl;
          if (HANDOFF) store_agent(entry + i, pack_sel_entry(p, sl));
          hmask[i] = 1;
          ++my_hits;
        } else {
          my_page[j] = p;
          ++my_misses;
        }
      }
    }
  }
  // one scan counts both: misses in the low half, hits in the high half (k <= 2048 each)
  int mh;
  const int packed_rank = fast_scan<NT>(my_misses | (my_hits << 16), sm, flip, mh);   // barrier inside: the hit bitmap is complete
  const int m = mh & 0xffff, n_hits = mh >> 16;
  int miss_rank = packed_rank & 0xffff;
  const int e = (R + m - C) > 0 ? (R + m - C) : 0;
  if (m == 0) {
    // every selected page is resident: no slot to find, nothing leaves, nothing to fetch
    for (int j = tid; j < k; j += NT) evout[j] = -1;
    if (tid == 0) {
      a.miss_count[u] = 0;
      a.counts[u * 3 + 0] = n_hits;
      a.counts[u * 3 + 1] = 0;
      a.counts[u * 3 + 2] = 0;
      atomicAdd(&a.stats[0], (unsigned long long)n_hits);
    }
    return true;
  }

  // ---- victims: the e smallest (stamp, page) among resident slots that were not hit
  auto is_cand = [&](int j) -> bool {
    const int sl = tid * CPT + j;
    return sp[j] >= 0 && !((sm.hit_bitmap[sl >> 5] >> (sl & 31)) & 1u);
  };
  u32 cand_mask = 0;
#pragma unroll
  for (int j = 0; j < CPT; ++j) cand_mask |= is_cand(j) ? (1u << j) : 0u;
  // lookahead eviction buckets the candidates' scores linearly between their extremes
  float vmin = 0.f, vinv = 0.f;
  if (a.lookahead && e > 0) {
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int j = 0; j < CPT; ++j)
      if (((cand_mask >> j) & 1u) && vs[j] > -INFINITY) {   // (a page of no cluster scores -inf: bucket 0 whatever the range)
        lo = fminf(lo, vs[j]);
        hi = fmaxf(hi, vs[j]);
      }
    lo = wave_allreduce_min(lo);
    hi = wave_allreduce_max(hi);
    if (lane == 0) { sm.red_min[w] = lo; sm.red_max[w] = hi; }
    __syncthreads();
    lo = sm.red_min[0]; hi = sm.red_max[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) {
      lo = fminf(lo, sm.red_min[i]);
      hi = fmaxf(hi, sm.red_max[i]);
    }
    vmin = lo;
    vinv = hi > lo ? 2047.0f / (hi - lo) : 0.f;
  }
  auto la_bucket = [&](float v) -> int { return (int)fminf(fmaxf((v - vmin) * vinv, 0.f), 2047.f); };
  // A finite look-ahead pool: the key of the pool's last member in selection order (best page first)
  // over the unit's valid pages; a resident page is in the pool iff its key is not beyond it.
  bool pooled = false;
  u64 pool_thr = ~0ull;
  if (a.lookahead && a.la_pool > 0 && e > 0) {
    int n_valid = (a.seq_len[b] + a.P - 1) / a.P;
    n_valid = n_valid < a.NP ? n_valid : a.NP;
    if (a.la_pool < n_valid) {
      pooled = true;
      auto fn = [&](int p, u64& kk) -> bool {
        kk = selection_order_key(victim_score<HANDOFF>(a, u, p), p);
        return true;
      };
      pool_thr = block_kth_smallest<NT>(fn, n_valid, a.la_pool, sm.generic, sm.a.sel.hist);
      // (the histogram serves the victim choice next: it must start from zero again)
      __syncthreads();
      for (int i = tid; i < kRadixBins; i += NT) sm.a.sel.hist[i] = 0;
      __syncthreads();
    }
  }
  auto in_pool = [&](float v, int page) -> bool { return selection_order_key(v, page) <= pool_thr; };
  auto la_key = [&](float v, int st, int page) -> u64 {
    return pooled ? pooled_victim_key(in_pool(v, page), v, st, page) : lookahead_victim_key(v, page);
  };
  auto la_bkt = [&](float v, int st, int page) -> int {
    if (!pooled) return la_bucket(v);
    // the halves of the bucket range: outside the pool by age, inside by score
    return in_pool(v, page) ? 1024 + (la_bucket(v) >> 1) : (victim_bucket((long long)a.step - (long long)st, page, a.NP) >> 1);
  };
  auto vkey_of = [&](int j) -> u64 {
    return a.lookahead ? la_key(vs[j], ss[j], sp[j]) : ((u64)((u32)ss[j] ^ 0x80000000u) << 32) | (u32)sp[j];
  };
  auto vbkt_of = [&](int j) -> int {
    if (!((cand_mask >> j) & 1u)) return -1;
    return a.lookahead ? la_bkt(vs[j], ss[j], sp[j]) : victim_bucket((long long)a.step - (long long)ss[j], sp[j], a.NP);
  };
  u64 vthr = 0;
  if (e > 0) {
    auto refine = [&](int bin, int r) -> u64 {
      auto fn = [&](int sl, u64& kk) -> bool {
        const int p = spage[sl];
        if (p < 0 || ((sm.hit_bitmap[sl >> 5] >> (sl & 31)) & 1u)) return false;
        const int st = sstamp[sl];
        if (a.lookahead) {
          const float v = victim_score<HANDOFF>(a, u, p);
          if (la_bkt(v, st, p) != bin) return false;
          kk = la_key(v, st, p);
          return true;
        }
        if (victim_bucket((long long)a.step - (long long)st, p, a.NP) != bin) return false;
        kk = ((u64)((u32)st ^ 0x80000000u) << 32) | (u32)p;
        return true;
      };
      return block_kth_smallest<NT>(fn, C, r, sm.generic, sm.a.sel.hist);
    };
    vthr = two_level_select<NT, CPT>(vkey_of, vbkt_of, e, sm, flip, refine);
  }

  // ---- hand out slots: free slots and victim slots in ascending slot order go to the misses in
  // ascending page order
  int avail = 0;
  u32 av_mask = 0, vic_mask = 0;
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const bool vic = e > 0 && ((cand_mask >> j) & 1u) && vkey_of(j) <= vthr;
    const bool av = sp[j] == -1 || vic;
    vic_mask |= vic ? (1u << j) : 0u;
    av_mask |= av ? (1u << j) : 0u;
    avail += av ? 1 : 0;
  }
  int total_avail;
  int rank = fast_scan<NT>(avail, sm, flip, total_avail);
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    if ((av_mask >> j) & 1u) {
      if (rank < m) {
        sm.assign[rank] = (uint16_t)(tid * CPT + j);
        if ((vic_mask >> j) & 1u) {
          const int at = atomicAdd(&sm.n_ev, 1);
          if (at < k) evout[at] = sp[j];
        }
      }
      ++rank;
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int p = my_page[j];
    if (p >= 0) {
      const int i = i0 + j;
      const int sl = sm.assign[miss_rank];
      const int slot = sl == kAbsent ? -1 : sl;       // always a slot while the directory is consistent
      sslots[i] = slot;
      my_slot[j] = slot;
      hmask[i] = 0;
      if (slot >= 0) {
        spage[slot] = p;
        sstamp[slot] = a.step;
      }
      a.miss_list[((size_t)u * k + miss_rank) * 2] = p;
      a.miss_list[((size_t)u * k + miss_rank) * 2 + 1] = slot;
      ++miss_rank;
    }
  }
  for (int j = e + tid; j < k; j += NT) evout[j] = -1;
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
  // the misses' entries go out when every wave's copies have been acknowledged
  auto publish_misses = [&]() {
    if (!HANDOFF) return;
    wave_drain_memory();
    __syncthreads();
#pragma unroll
    for (int j = 0; j < KPT; ++j)
      if (my_page[j] >= 0) store_agent(entry + i0 + j, pack_sel_entry(my_page[j], my_slot[j]));
  };
  if (!a.do_gather) {
    publish_misses();
    return true;
  }

  // ---- fetch the unit's missed pages: groups of 256 threads, one 16-token tile (or one page in
  // the natural layout) each per round.  Miss j is (page, sm.assign[j]); the pages are staged in
  // sm.sel[j], each thread writing the misses it found at their ranks.
  __syncthreads();                                     // everyone is done with sm.sel / sm.a.sel
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    // my misses keep their rank: miss_rank was advanced once per miss above
    const int p = my_page[KPT - 1 - j];
    if (p >= 0) sm.sel[--miss_rank] = (uint16_t)p;
  }
  __syncthreads();
  const int grp = tid >> 8, gt = tid & 255;
  const char* store_u = a.store + (size_t)u * a.NP * a.page_bytes;
  char* pool_u = a.pool + (size_t)u * a.Cmax * a.page_bytes;
  if (a.tiled == kLayoutPacked) {
    // pages of 4 or 8 tokens: one page per group and round
    for (int j0 = 0; j0 < m; j0 += kCopyGroups) {
      const int jm = j0 + grp;
      const bool on = jm < m;
      int page = 0, slot = -1;
      if (on) {
        page = sm.sel[jm];
        slot = sm.assign[jm] == kAbsent ? -1 : sm.assign[jm];
      }
      char* dst = pool_u + (size_t)(slot < 0 ? 0 : slot) * a.page_bytes;
      if (on && slot >= 0) packed_copy_phase_a<HANDOFF>(store_u + (size_t)page * a.page_bytes, a.P, dst, sm.a.vt[grp], gt);
      __syncthreads();
      if (on && slot >= 0) packed_copy_phase_b<HANDOFF>(a.P, dst, sm.a.vt[grp], gt);
      __syncthreads();
    }
  } else if (a.tiled) {
    const int tiles = a.P / kTileTokens;
    const int n_items = m * tiles;
    for (int it0 = 0; it0 < n_items; it0 += kCopyGroups) {
      const int it = it0 + grp;
      const bool on = it < n_items;
      int page = 0, slot = -1, tile = 0;
      if (on) {
        const int jm = it / tiles;
        tile = it % tiles;
        page = sm.sel[jm];
        slot = sm.assign[jm] == kAbsent ? -1 : sm.assign[jm];
      }
      char* dst_tile = pool_u + (size_t)(slot < 0 ? 0 : slot) * a.page_bytes + (size_t)tile * kTileBytes;
      if (on && slot >= 0) tile_copy_phase_a<HANDOFF>(store_u + (size_t)page * a.page_bytes, a.P, tile, dst_tile, sm.a.vt[grp], gt);
      __syncthreads();
      if (on && slot >= 0) tile_copy_phase_b<HANDOFF>(dst_tile, sm.a.vt[grp], gt);
      __syncthreads();
    }
  } else {
    const unsigned units = a.page_bytes / 16;
    for (int jm = grp; jm < m; jm += kCopyGroups) {
      const int page = sm.sel[jm];
      const int slot = sm.assign[jm] == kAbsent ? -1 : sm.assign[jm];
      if (slot < 0) continue;
      const uint4* s4 = reinterpret_cast<const uint4*>(store_u + (size_t)page * a.page_bytes);
      uint4* d4 = reinterpret_cast<uint4*>(pool_u + (size_t)slot * a.page_bytes);
      for (unsigned o = gt; o < units; o += 256) slot_store16<HANDOFF>(d4 + o, s4[o]);
    }
  }
  publish_misses();
  return true;
}

}  // namespace kvd
