// Selection through the hierarchical index (System Overview: the page means form higher-level
// centroids for similarity grouping): whole clusters are taken in (score descending, cluster
// ascending) order until the page budget is used up, the first cluster that does not fit giving its
// lowest pages; sink / recent pages are in first and are not counted as members of their clusters.
// Shared by the stand-alone kernel and the single-launch layer-step kernel.
#pragma once
#include "kvd_device.h"
#include "kvd_internal.h"

namespace kvd {

constexpr int kBitmapWordsCS = KVD_FAST_MAX_PAGES / 32;

template <int NT>
struct ClusterSelectSmem {
  u32 hist[kRadixBins];                  // pages per score bucket
  u32 bitmap[kBitmapWordsCS];            // selected pages
  u64 cand[KVD_MAX_CENTROIDS];           // clusters of the decisive bucket: score key << 32 | cluster << 16 | pages
  int scan[NT / kWave + 1];
  float red_min[NT / kWave], red_max[NT / kWave];
  int cand_n, bin, below;
};

__device__ __forceinline__ u32 cluster_descending_key(float s) {
  const u32 x = as_u32(s + 0.0f);                    // -0 -> +0 so that the two zeros tie
  const u32 asc = (x & 0x80000000u) ? ~x : (x | 0x80000000u);
  return ~asc;
}

// first index in [b, e) whose page is >= v (pages ascending)
__device__ __forceinline__ int lower_bound_pages(const int32_t* pages, int b, int e, int v) {
  while (b < e) {
    const int m = (b + e) >> 1;
    if (pages[m] < v) b = m + 1; else e = m;
  }
  return b;
}

// All NT threads of a workgroup, for unit u: scores [U][Nc] of the centroids -> sel_pages [U][k]
// ascending, -1 padded.  HANDOFF: the scores were written by other workgroups of the same launch
// and are read with device-scope loads.  Ends with every thread's part of sel_pages stored; a
// barrier is needed before other threads read it.
template <int NT, bool HANDOFF>
__device__ __forceinline__ void cluster_select_body(const float* __restrict__ scores, const int32_t* __restrict__ cluster_start,
                                                    const int32_t* __restrict__ cluster_pages, int32_t* __restrict__ sel_pages,
                                                    const int32_t* __restrict__ seq_len, int NP, int Nc, int P, int k, int sink,
                                                    int recent, int Hkv, int u, ClusterSelectSmem<NT>& sm) {
  constexpr int CPT = KVD_MAX_CENTROIDS / NT, NW = NT / kWave;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  int n_valid = (seq_len[u / Hkv] + P - 1) / P;
  n_valid = n_valid < NP ? n_valid : NP;
  // forced pages: [0, lo) and [hi, n_valid); members of clusters count only inside [lo, hi)
  const int lo = sink < n_valid ? sink : n_valid;
  int hi = n_valid - recent;
  hi = hi > lo ? hi : lo;
  const int n_forced = lo + (n_valid - hi);
  const int budget = k - n_forced;                      // >= 0: checked when the context was created
  const float* sc = scores + (size_t)u * Nc;
  const int32_t* start = cluster_start + (size_t)u * (Nc + 1);
  const int32_t* pages = cluster_pages + (size_t)u * NP;

  float s[CPT];
  int mb[CPT], size[CPT];                               // first counted member, number of counted members
  float fmin = INFINITY, fmax = -INFINITY;
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int c = tid + j * NT;                         // clusters interleaved over the threads
    s[j] = 0.f; mb[j] = 0; size[j] = 0;
    if (c < Nc) {
      s[j] = HANDOFF ? load_agent(sc + c) : sc[c];
      const int b = start[c], e = start[c + 1];
      if (n_forced == 0) {                              // no forced pages: every listed page counts
        mb[j] = b;
        size[j] = e - b;
      } else {
        mb[j] = lower_bound_pages(pages, b, e, lo);
        size[j] = lower_bound_pages(pages, mb[j], e, hi) - mb[j];
      }
      if (size[j] > 0) { fmin = fminf(fmin, s[j]); fmax = fmaxf(fmax, s[j]); }
    }
  }
  for (int i = tid; i < kRadixBins; i += NT) sm.hist[i] = 0;
  for (int i = tid; i < kBitmapWordsCS; i += NT) sm.bitmap[i] = 0;
  if (tid == 0) sm.cand_n = 0;
  fmin = wave_allreduce_min(fmin);
  fmax = wave_allreduce_max(fmax);
  if (lane == 0) { sm.red_min[w] = fmin; sm.red_max[w] = fmax; }
  __syncthreads();
  fmin = sm.red_min[0]; fmax = sm.red_max[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) { fmin = fminf(fmin, sm.red_min[i]); fmax = fmaxf(fmax, sm.red_max[i]); }
  const float range = fmax - fmin;
  const float inv = range > 0.f ? 2047.0f / range : 0.f;
  auto bucket_of = [&](float v) -> int { return (int)fminf(fmaxf((fmax - v) * inv, 0.f), 2047.f); };

  // pages per bucket; the bucket in which the running total passes the budget decides
#pragma unroll
  for (int j = 0; j < CPT; ++j)
    if (size[j] > 0) atomicAdd(&sm.hist[bucket_of(s[j])], (u32)size[j]);
  __syncthreads();
  constexpr int BPT = kRadixBins / NT;
  int local = 0;
#pragma unroll
  for (int j = 0; j < BPT; ++j) local += (int)sm.hist[tid * BPT + j];
  int total;
  int ex = block_exclusive_scan<NT>(local, sm.scan, total);
  if (tid == 0) { sm.bin = kRadixBins; sm.below = total; }   // everything fits unless some thread finds the crossing
  __syncthreads();
  if (total > budget && ex <= budget && budget < ex + local) {      // exactly one thread
    int b = tid * BPT;
    for (int j = 0; j < BPT; ++j, ++b) {
      const int cnt = (int)sm.hist[b];
      if (budget < ex + cnt) break;
      ex += cnt;
    }
    sm.bin = b;
    sm.below = ex;
  }
  __syncthreads();
  const int bin = sm.bin, below = sm.below;
  // clusters of the decisive bucket are ranked exactly
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    if (size[j] > 0 && bucket_of(s[j]) == bin) {
      const int at = atomicAdd(&sm.cand_n, 1);
      sm.cand[at] = ((u64)cluster_descending_key(s[j]) << 32) | ((u64)(tid + j * NT) << 16) | (u64)size[j];
    }
  }
  __syncthreads();
  const int m = sm.cand_n;
  // take[j]: pages taken from this thread's j-th cluster
  int take[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    take[j] = 0;
    if (size[j] > 0) {
      const int b = bucket_of(s[j]);
      if (b < bin) {
        take[j] = size[j];
      } else if (b == bin) {
        const u64 mine = (((u64)cluster_descending_key(s[j]) << 32) | ((u64)(tid + j * NT) << 16)) >> 16;
        int before = below;
        for (int x = 0; x < m; ++x) {
          const u64 other = sm.cand[x];
          before += (other >> 16) < mine ? (int)(other & 0xffffu) : 0;
        }
        const int room = budget - before;
        take[j] = room <= 0 ? 0 : (room < size[j] ? room : size[j]);
      }
    }
  }
  // mark: forced pages, then the taken members
  for (int p = tid; p < n_valid; p += NT)
    if (p < lo || p >= hi) atomicOr(&sm.bitmap[p >> 5], 1u << (p & 31));
#pragma unroll
  for (int j = 0; j < CPT; ++j)
    for (int i = 0; i < take[j]; ++i) {
      const int p = pages[mb[j] + i];
      atomicOr(&sm.bitmap[p >> 5], 1u << (p & 31));
    }
  __syncthreads();
  // compact in ascending page order: thread t owns bitmap words [t * WPT, (t+1) * WPT)
  constexpr int WPT = kBitmapWordsCS / NT > 0 ? kBitmapWordsCS / NT : 1;
  int cnt = 0;
  if (tid * WPT < kBitmapWordsCS) {
#pragma unroll
    for (int j = 0; j < WPT; ++j) cnt += __popc(sm.bitmap[tid * WPT + j]);
  }
  int n_sel;
  int pos = block_exclusive_scan<NT>(cnt, sm.scan, n_sel);
  int32_t* out = sel_pages + (size_t)u * k;
  if (tid * WPT < kBitmapWordsCS) {
#pragma unroll
    for (int j = 0; j < WPT; ++j) {
      u32 bits = sm.bitmap[tid * WPT + j];
      while (bits) {
        const int bit = __ffs((int)bits) - 1;
        bits &= bits - 1;
        if (pos < k) out[pos] = (tid * WPT + j) * 32 + bit;
        ++pos;
      }
    }
  }
  for (int i = n_sel + tid; i < k; i += NT) out[i] = -1;
}

}  // namespace kvd
