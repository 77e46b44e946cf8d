// Stage 3 of the decode step: GQA decode attention over the selected pages only (System
// Overview: attention runs over the union of resident and newly fetched entries).  The selected
// pages of a unit are split over several blocks (split-K); each block streams its K/V pages from
// the slot pool once, keeps an fp32 online softmax per query head, and the partial results are
// merged by log-sum-exp.
#include "kvd_device.h"
#include "kvd_internal.h"

namespace kvd {

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
  const uint16_t* q;         // [B][Hq][D]
  const char* pool;          // [U][Cmax] slots of the layer
  const int32_t* sel_pages;  // [U][k]
  const int32_t* sel_slots;  // [U][k]
  const int32_t* seq_len;    // [B]
  float* part_acc;           // [U][S][G][D]
  float* part_ml;            // [U][S][G][2]
  int k, P, Cmax, Hq, Hkv, S, per_split;
  unsigned page_bytes;
  float scale_log2;          // softmax scale * log2(e)
};

// Block (split, u): 4 waves, wave w takes selected entries first + w, first + w + 4, ...
// A wave load covers 4 token rows: lane (r, c) = (lane / 16, lane % 16) holds dims 8c..8c+7 of
// token 4j + r of a 16-token tile.  Each 16-lane row keeps its own running (max, sum, acc) for the
// G query heads, so nothing crosses rows inside the loop; rows and waves are merged at the end.
template <bool BF16, int G>
__global__ __launch_bounds__(kAttnThreads) void attend_kernel(AttnArgs a) {
  __shared__ float sh_acc[kAttnWaves][G][kHeadDim];
  __shared__ float sh_m[kAttnWaves][G];
  __shared__ float sh_l[kAttnWaves][G];
  const int split = blockIdx.x, u = blockIdx.y;
  const int b = u / a.Hkv, h = u % a.Hkv;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int r = lane >> 4, c = lane & 15;

  float qf[G][8];
  {
    const uint16_t* qrow = a.q + ((size_t)b * a.Hq + (size_t)h * G) * kHeadDim + c * 8;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const uint4 raw = *reinterpret_cast<const uint4*>(qrow + (size_t)g * kHeadDim);
      cvt8<BF16>(raw, qf[g]);
    }
  }
  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  }

  const int seq = a.seq_len[b];
  const int first = split * a.per_split;
  const int last = (first + a.per_split) < a.k ? (first + a.per_split) : a.k;
  const int32_t* sel = a.sel_pages + (size_t)u * a.k;
  const int32_t* slots = a.sel_slots + (size_t)u * a.k;
  const char* pool_u = a.pool + (size_t)u * a.Cmax * a.page_bytes;

  for (int i = first + w; i < last; i += kAttnWaves) {
    const int page = __builtin_amdgcn_readfirstlane(sel[i]);
    const int slot = __builtin_amdgcn_readfirstlane(slots[i]);
    if (page < 0 || slot < 0 || slot >= a.Cmax) continue;
    int ntok = seq - page * a.P;
    ntok = ntok < a.P ? ntok : a.P;
    if (ntok <= 0) continue;
    const char* kbase = pool_u + (size_t)slot * a.page_bytes + c * 16;
    const char* vbase = kbase + (size_t)a.P * kRowBytes;
    for (int t0 = 0; t0 < ntok; t0 += 16) {
      uint4 kraw[4], vraw[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int tok = t0 + 4 * j + r;
        tok = tok < ntok ? tok : ntok - 1;
        kraw[j] = *reinterpret_cast<const uint4*>(kbase + (size_t)tok * kRowBytes);
        vraw[j] = *reinterpret_cast<const uint4*>(vbase + (size_t)tok * kRowBytes);
      }
      float x[4][G];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float kf[8];
        cvt8<BF16>(kraw[j], kf);
        const bool valid = (t0 + 4 * j + r) < ntok;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float s = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) s = fmaf(qf[g][e], kf[e], s);
          s = row16_allreduce_sum(s);
          x[j][g] = valid ? s * a.scale_log2 : -INFINITY;
        }
      }
      float p[4][G];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mx = fmaxf(fmaxf(x[0][g], x[1][g]), fmaxf(x[2][g], x[3][g]));
        const float m_new = fmaxf(m[g], mx);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m[g] - m_safe);
        float ps = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          p[j][g] = exp2f(x[j][g] - m_safe);
          ps += p[j][g];
        }
        l[g] = l[g] * alpha + ps;
        m[g] = m_new;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float vf[8];
        cvt8<BF16>(vraw[j], vf);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(p[j][g], vf[e], acc[g][e]);
      }
    }
  }

  // merge the 4 rows of the wave (lanes differing in bits 4 and 5)
#pragma unroll
  for (int g = 0; g < G; ++g) {
#pragma unroll
    for (int mask = 16; mask <= 32; mask <<= 1) {
      const float mo = __shfl_xor(m[g], mask, kWave);
      const float lo = __shfl_xor(l[g], mask, kWave);
      const float mn = fmaxf(m[g], mo);
      const float ms = mn == -INFINITY ? 0.f : mn;
      const float sa = exp2f(m[g] - ms), sb = exp2f(mo - ms);
      l[g] = l[g] * sa + lo * sb;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float ao = __shfl_xor(acc[g][e], mask, kWave);
        acc[g][e] = acc[g][e] * sa + ao * sb;
      }
      m[g] = mn;
    }
  }
  if (r == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sh_acc[w][g][c * 8 + e] = acc[g][e];
      if (c == 0) { sh_m[w][g] = m[g]; sh_l[w][g] = l[g]; }
    }
  }
  __syncthreads();
  // merge the 4 waves and write this split's partial result
  for (int idx = tid; idx < G * kHeadDim; idx += kAttnThreads) {
    const int g = idx / kHeadDim, d = idx % kHeadDim;
    float M = sh_m[0][g];
#pragma unroll
    for (int ww = 1; ww < kAttnWaves; ++ww) M = fmaxf(M, sh_m[ww][g]);
    const float Ms = M == -INFINITY ? 0.f : M;
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int ww = 0; ww < kAttnWaves; ++ww) {
      const float sc = exp2f(sh_m[ww][g] - Ms);
      L += sh_l[ww][g] * sc;
      A += sh_acc[ww][g][d] * sc;
    }
    const size_t base = ((size_t)u * a.S + split) * G + g;
    a.part_acc[base * kHeadDim + d] = A;
    if (d == 0) {
      a.part_ml[base * 2] = M;
      a.part_ml[base * 2 + 1] = L;
    }
  }
}

// Merge of the S split partials of a unit: one block per unit, one thread per output dimension.
__global__ __launch_bounds__(kHeadDim) void combine_kernel(const float* __restrict__ part_acc,
                                                          const float* __restrict__ part_ml, float* __restrict__ out,
                                                          float* __restrict__ lse, int S, int G, int Hq, int Hkv) {
  const int u = blockIdx.x, d = threadIdx.x;
  const int b = u / Hkv, h = u % Hkv;
  for (int g = 0; g < G; ++g) {
    float M = -INFINITY;
    for (int s = 0; s < S; ++s) M = fmaxf(M, part_ml[(((size_t)u * S + s) * G + g) * 2]);
    const float Ms = M == -INFINITY ? 0.f : M;
    float L = 0.f, A = 0.f;
    for (int s = 0; s < S; ++s) {
      const size_t base = ((size_t)u * S + s) * G + g;
      const float sc = exp2f(part_ml[base * 2] - Ms);
      L += part_ml[base * 2 + 1] * sc;
      A += part_acc[base * kHeadDim + d] * sc;
    }
    const size_t row = (size_t)b * Hq + (size_t)h * G + g;
    out[row * kHeadDim + d] = A / L;
    if (lse != nullptr && d == 0) lse[row] = (M + log2f(L)) * kLn2;
  }
}

template <bool BF16, int G>
static void launch_attend(const AttnArgs& a, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL((attend_kernel<BF16, G>), grid, dim3(kAttnThreads), 0, s, a);
}

template <bool BF16>
static bool dispatch_group(int G, const AttnArgs& a, dim3 grid, hipStream_t s) {
  switch (G) {
    case 1: launch_attend<BF16, 1>(a, grid, s); return true;
    case 2: launch_attend<BF16, 2>(a, grid, s); return true;
    case 3: launch_attend<BF16, 3>(a, grid, s); return true;
    case 4: launch_attend<BF16, 4>(a, grid, s); return true;
    case 5: launch_attend<BF16, 5>(a, grid, s); return true;
    case 6: launch_attend<BF16, 6>(a, grid, s); return true;
    case 7: launch_attend<BF16, 7>(a, grid, s); return true;
    case 8: launch_attend<BF16, 8>(a, grid, s); return true;
    default: return false;
  }
}

}  // namespace kvd

hipError_t kvd_launch_attend(kvd_ctx* c, int layer, const void* q, const int32_t* sel_pages,
                             const int32_t* sel_slots, hipStream_t s) {
  using namespace kvd;
  AttnArgs a;
  a.q = reinterpret_cast<const uint16_t*>(q);
  a.pool = c->pool + (size_t)layer * c->U * c->Cmax * c->page_bytes;
  a.sel_pages = sel_pages;
  a.sel_slots = sel_slots;
  a.seq_len = c->d_seq_len;
  a.part_acc = c->d_part_acc;
  a.part_ml = c->d_part_ml;
  a.k = c->k; a.P = c->P; a.Cmax = c->Cmax; a.Hq = c->Hq; a.Hkv = c->Hkv; a.S = c->S;
  a.per_split = (c->k + c->S - 1) / c->S;
  a.page_bytes = (unsigned)c->page_bytes;
  a.scale_log2 = c->scale * kLog2e;
  dim3 grid(c->S, c->U);
  const bool ok = c->bf16 ? dispatch_group<true>(c->G, a, grid, s) : dispatch_group<false>(c->G, a, grid, s);
  if (!ok) return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t kvd_launch_combine(kvd_ctx* c, float* out, float* lse, hipStream_t s) {
  using namespace kvd;
  hipLaunchKernelGGL(combine_kernel, dim3(c->U), dim3(kHeadDim), 0, s, c->d_part_acc, c->d_part_ml, out, lse, c->S,
                     c->G, c->Hq, c->Hkv);
  return hipGetLastError();
}
