// Scoring of page summaries against the pooled query, one wave at a time (Background, "KV Cache
// Offloading": the query is multiplied with the index representatives; System Overview: the
// representative is the page's mean key).  Shared by the stand-alone scoring kernel and by the
// single-launch layer-step kernel.
#pragma once
#include "kvd_device.h"

namespace kvd {

// One wave scores pages [wave_base, wave_base + 64 * passes) of one unit in passes of 64.  A wave
// load covers 4 summary rows (4 x 256 B): lane (r, c) = (lane / 16, lane % 16) holds dims
// 8c..8c+7 of row r.  The 16 partial dot products of a row are summed with DPP row rotations;
// after 16 loads lane (r, c) keeps the score of page base + 4c + r and the wave stores 64
// consecutive scores.  The first summary loads are issued before the query is fetched, so the
// wave does not sit idle for a round trip before it starts streaming.
//   summ_u   [NP][D]  summaries of the unit
//   q_group  [G][D]   the unit's G query heads
//   scores_u [NP]
// HANDOFF: the scores are consumed by another workgroup of the same launch, so they are stored
// with device-scope write-through stores.
template <bool BF16, bool HANDOFF>
__device__ __forceinline__ void score_wave(const uint16_t* __restrict__ summ_u, const uint16_t* __restrict__ q_group,
                                           float* __restrict__ scores_u, int NP, int G, float scale, int wave_base,
                                           int passes) {
  const int lane = threadIdx.x & (kWave - 1);
  const int r = lane >> 4, c = lane & 15;
  if (wave_base >= NP) return;
  const uint16_t* srow = summ_u + c * 8;

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
  const uint16_t* qrow = q_group + c * 8;
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
    if (page < NP) {
      if (HANDOFF) store_agent(scores_u + page, mine * scale);
      else scores_u[page] = mine * scale;
    }
  }
}

}  // namespace kvd
