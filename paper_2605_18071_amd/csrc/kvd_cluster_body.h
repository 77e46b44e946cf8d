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

// What a thread knows of its clusters before any score is there: the first counted member and the
// number of counted members of cluster tid + j * NT (counted: inside [lo, hi), i.e. not a sink or
// recent page).
template <int NT>
struct ClusterPrep {
  static constexpr int CPT = KVD_MAX_CENTROIDS / NT;
  int mb[CPT], size[CPT];
  int n_valid, lo, hi, n_forced, budget;
};

// All NT threads of a workgroup, for unit u: everything the selection needs that does not depend
// on this step's scores (the cluster bounds, and with sink / recent pages the searches in the
// members' lists).  A caller that has to wait for the scores calls this before it waits.
template <int NT>
__device__ __forceinline__ void cluster_prepare(const int32_t* __restrict__ cluster_start, const int32_t* __restrict__ cluster_pages,
                                                const int32_t* __restrict__ seq_len, int NP, int Nc, int P, int k, int sink,
                                                int recent, int Hkv, int u, ClusterPrep<NT>& pr) {
  constexpr int CPT = ClusterPrep<NT>::CPT;
  const int tid = threadIdx.x;
  int n_valid = (seq_len[u / Hkv] + P - 1) / P;
  n_valid = n_valid < NP ? n_valid : NP;
  // forced pages: [0, lo) and [hi, n_valid); members of clusters count only inside [lo, hi)
  const int lo = sink < n_valid ? sink : n_valid;
  int hi = n_valid - recent;
  hi = hi > lo ? hi : lo;
  pr.n_valid = n_valid; pr.lo = lo; pr.hi = hi;
  pr.n_forced = lo + (n_valid - hi);
  pr.budget = k - pr.n_forced;                          // >= 0: checked when the context was created
  const int32_t* start = cluster_start + (size_t)u * (Nc + 1);
  const int32_t* pages = cluster_pages + (size_t)u * NP;
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int c = tid + j * NT;                         // clusters interleaved over the threads
    pr.mb[j] = 0; pr.size[j] = 0;
    if (c < Nc) {
      const int b = start[c], e = start[c + 1];
      if (pr.n_forced == 0) {                           // no forced pages: every listed page counts
        pr.mb[j] = b;
        pr.size[j] = e - b;
      } else {
        pr.mb[j] = lower_bound_pages(pages, b, e, lo);
        pr.size[j] = lower_bound_pages(pages, pr.mb[j], e, hi) - pr.mb[j];
      }
    }
  }
}

// All NT threads of a workgroup, for unit u: scores [U][Nc] of the centroids -> sel_pages [U][k]
// ascending, -1 padded, and, if sel_lds is given, the same selection as 16-bit pages in LDS
// (0xffff = padding) for a directory update by the same workgroup.  HANDOFF: the scores were
// written by other workgroups of the same launch and are read with device-scope loads.  Ends
// with every thread's part of the selection stored; a barrier is needed before other threads read it.
template <int NT, bool HANDOFF>
__device__ __forceinline__ void cluster_finish(const float* __restrict__ scores, const int32_t* __restrict__ cluster_pages,
                                               int32_t* __restrict__ sel_pages, uint16_t* sel_lds, int NP, int Nc, int k, int u,
                                               const ClusterPrep<NT>& pr, ClusterSelectSmem<NT>& sm) {
  constexpr int CPT = ClusterPrep<NT>::CPT, NW = NT / kWave;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int n_valid = pr.n_valid, lo = pr.lo, hi = pr.hi, budget = pr.budget;
  const float* sc = scores + (size_t)u * Nc;
  const int32_t* pages = cluster_pages + (size_t)u * NP;

  float s[CPT];
  float fmin = INFINITY, fmax = -INFINITY;
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int c = tid + j * NT;
    s[j] = 0.f;
    if (c < Nc) s[j] = HANDOFF ? load_agent(sc + c) : sc[c];
  }
  for (int i = tid; i < kRadixBins; i += NT) sm.hist[i] = 0;
  for (int i = tid; i < kBitmapWordsCS; i += NT) sm.bitmap[i] = 0;
  if (tid == 0) sm.cand_n = 0;
#pragma unroll
  for (int j = 0; j < CPT; ++j)
    if (pr.size[j] > 0) { fmin = fminf(fmin, s[j]); fmax = fmaxf(fmax, s[j]); }
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
    if (pr.size[j] > 0) atomicAdd(&sm.hist[bucket_of(s[j])], (u32)pr.size[j]);
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
    if (pr.size[j] > 0 && bucket_of(s[j]) == bin) {
      const int at = atomicAdd(&sm.cand_n, 1);
      sm.cand[at] = ((u64)cluster_descending_key(s[j]) << 32) | ((u64)(tid + j * NT) << 16) | (u64)pr.size[j];
    }
  }
  __syncthreads();
  const int m = sm.cand_n;
  // take[j]: pages taken from this thread's j-th cluster
  int take[CPT];
  int my_clusters = 0, my_pages = 0;
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    take[j] = 0;
    if (pr.size[j] > 0) {
      const int b = bucket_of(s[j]);
      if (b < bin) {
        take[j] = pr.size[j];
      } else if (b == bin) {
        const u64 mine = (((u64)cluster_descending_key(s[j]) << 32) | ((u64)(tid + j * NT) << 16)) >> 16;
        int before = below;
        for (int x = 0; x < m; ++x) {
          const u64 other = sm.cand[x];
          before += (other >> 16) < mine ? (int)(other & 0xffffu) : 0;
        }
        const int room = budget - before;
        take[j] = room <= 0 ? 0 : (room < pr.size[j] ? room : pr.size[j]);
      }
    }
    my_clusters += take[j] > 0 ? 1 : 0;
    my_pages += take[j];
  }
  // The taken clusters as one list (first member, first output position) in what was the
  // candidates' array: one packed scan gives every thread its place in the list (high half) and its
  // first output position (low half); both stay below 2^15 (at most k <= 2048 pages are taken, at
  // least one from each taken cluster).
  int packed_total;
  const int packed = block_exclusive_scan<NT>((my_clusters << 16) | my_pages, sm.scan, packed_total);   // (barriers inside: the candidates have been read)
  const int n_list = packed_total >> 16, n_taken = packed_total & 0xffff;
  int32_t* list_first = reinterpret_cast<int32_t*>(sm.cand);           // [n_list]
  int32_t* list_pos = list_first + KVD_MAX_TOPK;                        // [n_list + 1]
  {
    int at = packed >> 16, pos = packed & 0xffff;
#pragma unroll
    for (int j = 0; j < CPT; ++j)
      if (take[j] > 0) {
        list_first[at] = pr.mb[j];
        list_pos[at] = pos;
        ++at;
        pos += take[j];
      }
    if (tid == 0) list_pos[n_list] = n_taken;
  }
  // mark the forced pages meanwhile
  for (int p = tid; p < n_valid; p += NT)
    if (p < lo || p >= hi) atomicOr(&sm.bitmap[p >> 5], 1u << (p & 31));
  __syncthreads();
  // every taken page by one thread: its cluster by bisection of the output positions, then one
  // independent load from the cluster's member list
  for (int i = tid; i < n_taken; i += NT) {
    int a0 = 0, a1 = n_list - 1;
    while (a0 < a1) {
      const int mid = (a0 + a1 + 1) >> 1;
      if (list_pos[mid] <= i) a0 = mid; else a1 = mid - 1;
    }
    const int p = pages[list_first[a0] + (i - list_pos[a0])];
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
        if (pos < k) {
          const int p = (tid * WPT + j) * 32 + bit;
          out[pos] = p;
          if (sel_lds != nullptr) sel_lds[pos] = (uint16_t)p;
        }
        ++pos;
      }
    }
  }
  for (int i = n_sel + tid; i < k; i += NT) {
    out[i] = -1;
    if (sel_lds != nullptr) sel_lds[i] = 0xffffu;
  }
}

// Both halves back to back, for a caller whose scores are already there.
template <int NT, bool HANDOFF>
__device__ __forceinline__ void cluster_select_body(const float* __restrict__ scores, const int32_t* __restrict__ cluster_start,
                                                    const int32_t* __restrict__ cluster_pages, int32_t* __restrict__ sel_pages,
                                                    const int32_t* __restrict__ seq_len, int NP, int Nc, int P, int k, int sink,
                                                    int recent, int Hkv, int u, ClusterSelectSmem<NT>& sm) {
  ClusterPrep<NT> pr;
  cluster_prepare<NT>(cluster_start, cluster_pages, seq_len, NP, Nc, P, k, sink, recent, Hkv, u, pr);
  cluster_finish<NT, HANDOFF>(scores, cluster_pages, sel_pages, nullptr, NP, Nc, k, u, pr, sm);
}

}  // namespace kvd
