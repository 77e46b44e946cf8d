// Stage 1 of the decode step: score every page summary against the pooled query, then keep the
// Top-K pages (Background, "KV Cache Offloading": the query is multiplied with the index
// representatives and the Top-K retrieved; System Overview: the representative is the page's
// mean key).  Scoring streams the index once and is bound by HBM bandwidth; selection is an
// exact radix refinement in LDS on (score descending, page ascending) keys.
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_score_body.h"

namespace kvd {

constexpr int kScoreThreads = 256;
constexpr int kScoreWaves = kScoreThreads / kWave;

// One block scores 256 * passes consecutive pages of one unit, each of its 4 waves 64 * passes of
// them (see score_wave).
template <bool BF16>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const uint16_t* __restrict__ summ,  // [U][NP][D] of the layer
                                                             const uint16_t* __restrict__ q,     // [B][Hq][D]
                                                             float* __restrict__ scores,         // [U][NP]
                                                             int NP, int G, int Hq, int Hkv, float scale, int u0, int passes) {
  const int u = blockIdx.y + u0;
  const int b = u / Hkv, h = u % Hkv;
  const int w = threadIdx.x / kWave;
  const int wave_base = (blockIdx.x * kScoreWaves + w) * 64 * passes;
  score_wave<BF16, false>(summ + (size_t)u * NP * kHeadDim, q + ((size_t)b * Hq + (size_t)h * G) * kHeadDim,
                          scores + (size_t)u * NP, NP, G, scale, wave_base, passes);
}

constexpr int kSelectThreads = 1024;

// Order-preserving map of a float to an unsigned key that *descends* with the score.
__device__ __forceinline__ u32 descending_key(float s) {
  const u32 x = as_u32(s + 0.0f);                 // -0 -> +0 so that the two zeros tie
  const u32 asc = (x & 0x80000000u) ? ~x : (x | 0x80000000u);
  return ~asc;
}

// One block per unit: exact Top-K with ties to the lower page.  Every page gets the distinct
// 64-bit key (descending_key(score) << 32 | page); forced pages (sink / recent) get the smallest
// possible high word.  The k-th smallest key is the threshold; pages at or below it are written
// in ascending page order.
__global__ __launch_bounds__(kSelectThreads) void select_kernel(const float* __restrict__ scores,   // [U][NP]
                                                               int32_t* __restrict__ sel_pages,    // [U][k]
                                                               const int32_t* __restrict__ seq_len,
                                                               int NP, int P, int k, int sink, int recent, int Hkv,
                                                               int u0) {
  __shared__ SelectSmem sm;
  __shared__ u32 radix_hist[kRadixBins];
  const int u = blockIdx.x + u0;
  const int b = u / Hkv;
  const int tid = threadIdx.x;
  int n_valid = (seq_len[b] + P - 1) / P;
  n_valid = n_valid < NP ? n_valid : NP;
  const int k_eff = k < n_valid ? k : n_valid;
  const float* sc = scores + (size_t)u * NP;
  int32_t* out = sel_pages + (size_t)u * k;
  const int recent_from = n_valid - recent;

  auto keyfn = [&](int i, u64& key) -> bool {
    const bool forced = i < sink || i >= recent_from;
    const u32 hi = forced ? 0u : descending_key(sc[i]);
    key = ((u64)hi << 32) | (u32)i;
    return true;
  };
  const u64 thr = block_kth_smallest<kSelectThreads>(keyfn, n_valid, k_eff, sm, radix_hist);

  const int per = (n_valid + kSelectThreads - 1) / kSelectThreads;   // consecutive pages per thread
  const int p0 = tid * per;
  const int p1 = (p0 + per) < n_valid ? (p0 + per) : n_valid;
  int cnt = 0;
  for (int p = p0; p < p1; ++p) {
    u64 key;
    keyfn(p, key);
    cnt += key <= thr ? 1 : 0;
  }
  int total;
  int pos = block_exclusive_scan<kSelectThreads>(cnt, sm.scan, total);
  for (int p = p0; p < p1; ++p) {
    u64 key;
    keyfn(p, key);
    if (key <= thr) {
      if (pos < k) out[pos] = p;
      ++pos;
    }
  }
  for (int j = k_eff + tid; j < k; j += kSelectThreads) out[j] = -1;
}

}  // namespace kvd

hipError_t kvd_launch_score(kvd_ctx* c, int layer, const void* q, float* scores, int u0, int u1, hipStream_t s) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  // the index that is scored: the page summaries, or the centroids of the hierarchical index
  const int NP = c->Nc > 0 ? c->Nc : c->NP;
  const uint16_t* summ = reinterpret_cast<const uint16_t*>(c->Nc > 0 ? c->centroids : c->summaries) + (size_t)layer * c->U * NP * kHeadDim;
  // about c->score_blocks blocks in total, so that the grid is one round of resident blocks
  const int n_units = u1 - u0;
  const long long pages = (long long)NP * n_units;
  int passes = (int)((pages + 256LL * c->score_blocks - 1) / (256LL * c->score_blocks));
  if (passes < 1) passes = 1;
  const int per_block = 256 * passes;
  dim3 grid((NP + per_block - 1) / per_block, n_units);
  if (c->bf16)
    hipLaunchKernelGGL(score_kernel<true>, grid, dim3(kScoreThreads), 0, s, summ, (const uint16_t*)q, scores, NP,
                       c->G, c->Hq, c->Hkv, c->scale, u0, passes);
  else
    hipLaunchKernelGGL(score_kernel<false>, grid, dim3(kScoreThreads), 0, s, summ, (const uint16_t*)q, scores, NP,
                       c->G, c->Hq, c->Hkv, c->scale, u0, passes);
  return hipGetLastError();
}

hipError_t kvd_launch_select(kvd_ctx* c, const float* scores, int32_t* sel_pages, int u0, int u1, hipStream_t s) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  hipLaunchKernelGGL(select_kernel, dim3(u1 - u0), dim3(kSelectThreads), 0, s, scores, sel_pages, c->d_seq_len, c->NP,
                     c->P, c->k, c->cfg.sink_pages, c->cfg.recent_pages, c->Hkv, u0);
  return hipGetLastError();
}
