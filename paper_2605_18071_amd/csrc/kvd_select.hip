// Stage 1 of the decode step: score every page summary against the pooled query, then keep the
// Top-K pages (Background, "KV Cache Offloading": the query is multiplied with the index
// representatives and the Top-K retrieved; System Overview: the representative is the page's
// mean key).  Scoring streams the index once and is bound by HBM bandwidth; selection is an
// exact radix refinement in LDS on (score descending, page ascending) keys.
#include "kvd_device.h"
#include "kvd_internal.h"

namespace kvd {

constexpr int kScoreThreads = 256;
constexpr int kScoreWaves = kScoreThreads / kWave;

// One block scores 256 * passes consecutive pages of one unit, each wave 64 * passes of them in
// passes of 64.  A wave
// load covers 4 summary rows (4 x 256 B): lane (r, c) = (lane / 16, lane % 16) holds dims
// 8c..8c+7 of row r.  The 16 partial dot products of a row are summed with DPP row rotations;
// after 16 loads lane (r, c) keeps the score of page base + 4c + r and the wave stores 64
// consecutive scores.  The first summary loads are issued before the query is fetched, so the
// block does not sit idle for a round trip before it starts streaming.
template <bool BF16>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const uint16_t* __restrict__ summ,  // [U][NP][D] of the layer
                                                             const uint16_t* __restrict__ q,     // [B][Hq][D]
                                                             float* __restrict__ scores,         // [U][NP]
                                                             int NP, int G, int Hq, int Hkv, float scale, int u0, int passes) {
  const int u = blockIdx.y + u0;
  const int b = u / Hkv, h = u % Hkv;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int r = lane >> 4, c = lane & 15;
  const int wave_base = (blockIdx.x * kScoreWaves + w) * 64 * passes;
  if (wave_base >= NP) return;
  const uint16_t* srow = summ + (size_t)u * NP * kHeadDim + c * 8;

  uint4 raw[8];
  auto issue = [&](int base, int half) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int page = base + 4 * (half * 8 + i) + r;
      page = page < NP ? page : NP - 1;
      raw[i] = load_stream16(srow + (size_t)page * kHeadDim);
    }
  };
  issue(wave_base, 0);

  float qbar[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) qbar[e] = 0.f;
  const uint16_t* qrow = q + ((size_t)b * Hq + (size_t)h * G) * kHeadDim + c * 8;
  for (int g = 0; g < G; ++g) {
    const uint4 qraw = *reinterpret_cast<const uint4*>(qrow + (size_t)g * kHeadDim);
    float f[8];
    cvt8<BF16>(qraw, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) qbar[e] += f[e];
  }
  const float fg = (float)G;
#pragma unroll
  for (int e = 0; e < 8; ++e) qbar[e] = qbar[e] / fg;

  for (int pass = 0; pass < passes; ++pass) {
    const int base = wave_base + pass * 64;
    if (base >= NP) break;
    float mine = 0.f;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      uint4 cur[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) cur[i] = raw[i];
      // next batch in flight while this one is reduced
      if (half == 0) issue(base, 1);
      else if (pass + 1 < passes && base + 64 < NP) issue(base + 64, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float f[8];
        cvt8<BF16>(cur[i], f);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(qbar[e], f[e], acc);
        acc = row16_allreduce_sum(acc);
        if (c == half * 8 + i) mine = acc;
      }
    }
    const int page = base + 4 * c + r;
    if (page < NP) scores[(size_t)u * NP + page] = mine * scale;
  }
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
  const uint16_t* summ = reinterpret_cast<const uint16_t*>(c->summaries) + (size_t)layer * c->U * c->NP * kHeadDim;
  // about c->score_blocks blocks in total, so that the grid is one round of resident blocks
  const int n_units = u1 - u0;
  const long long pages = (long long)c->NP * n_units;
  int passes = (int)((pages + 256LL * c->score_blocks - 1) / (256LL * c->score_blocks));
  if (passes < 1) passes = 1;
  const int per_block = 256 * passes;
  dim3 grid((c->NP + per_block - 1) / per_block, n_units);
  if (c->bf16)
    hipLaunchKernelGGL(score_kernel<true>, grid, dim3(kScoreThreads), 0, s, summ, (const uint16_t*)q, scores, c->NP,
                       c->G, c->Hq, c->Hkv, c->scale, u0, passes);
  else
    hipLaunchKernelGGL(score_kernel<false>, grid, dim3(kScoreThreads), 0, s, summ, (const uint16_t*)q, scores, c->NP,
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
