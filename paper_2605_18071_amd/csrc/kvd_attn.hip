// Stage 3 of the decode step: GQA decode attention over the selected pages only (System
// Overview: attention runs over the union of resident and newly fetched entries).  The selected
// pages of a unit are split over several blocks (split-K); each block streams its K/V pages from
// the slot pool once and keeps an fp32 online softmax per query head; the last block of a unit to
// finish merges the split partials by log-sum-exp and writes the output.
//
// Two kernels share that frame:
//  * attend_mfma_kernel — pages whose size is a multiple of 16 tokens are kept in the slot pool in
//    an operand-ready tile layout (see kvd_tile_layout.h), so that every wave load is 1 KiB
//    contiguous and lands directly in MFMA operand registers: S^T = K Q^T with 16x16x32 MFMAs,
//    O^T += V^T P^T with 16x16x16 MFMAs whose B operand is the softmaxed C tile of the first.
//  * attend_valu_kernel — any page size, natural [token][dim] slots, fp32 VALU arithmetic.
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_tile_layout.h"

namespace kvd {

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr int kAttnIdxCap = 512;          // (page, slot) entries of a split kept in LDS
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
  int32_t* ticket;           // [U], zero between launches
  float* out;                // [B][Hq][D]
  float* lse;                // [B][Hq] or null
  int k, P, Cmax, Hq, Hkv, S, per_split, fuse_merge, u0;
  unsigned page_bytes;
  float scale_log2;          // softmax scale * log2(e)
};

template <int G>
struct AttnSmem {
  float acc[kAttnWaves][G][kHeadDim];
  float m[kAttnWaves][G];
  float l[kAttnWaves][G];
  int is_last;
};

// Log-sum-exp merge of the S split partials of unit u into out / lse, by one block.  The
// partials are fetched in batches of 8 splits whose loads are all issued before any is used.
template <int G>
__device__ __forceinline__ void merge_splits(const AttnArgs& a, int u) {
  const int tid = threadIdx.x;
  const int b = u / a.Hkv, h = u % a.Hkv;
  for (int idx = tid; idx < G * kHeadDim; idx += kAttnThreads) {
    const int g = idx / kHeadDim, d = idx % kHeadDim;
    const float2* ml = reinterpret_cast<const float2*>(a.part_ml) + ((size_t)u * a.S * G + g);
    const float* pa = a.part_acc + ((size_t)u * a.S * G + g) * kHeadDim + d;
    float M = -INFINITY, L = 0.f, A = 0.f;
    for (int s0 = 0; s0 < a.S; s0 += 8) {
      float2 mlv[8];
      float av[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int s = (s0 + i) < a.S ? (s0 + i) : (a.S - 1);
        mlv[i] = ml[(size_t)s * G];
        av[i] = pa[(size_t)s * G * kHeadDim];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (s0 + i < a.S) {
          const float Mn = fmaxf(M, mlv[i].x);
          const float Ms = Mn == -INFINITY ? 0.f : Mn;
          const float so = exp2f(M - Ms), sn = exp2f(mlv[i].x - Ms);
          L = L * so + mlv[i].y * sn;
          A = A * so + av[i] * sn;
          M = Mn;
        }
      }
    }
    const size_t row = (size_t)b * a.Hq + (size_t)h * G + g;
    a.out[row * kHeadDim + d] = A / L;
    if (a.lse != nullptr && d == 0) a.lse[row] = (M + log2f(L)) * kLn2;
  }
}

// Block epilogue.  The waves have left their (max, sum, acc) in `sm`; merge them, write this
// split's partial, and let the last split of the unit to arrive merge all S partials.
template <int G>
__device__ __forceinline__ void finish_split(const AttnArgs& a, AttnSmem<G>& sm, int u, int split) {
  const int tid = threadIdx.x;
  const int b = u / a.Hkv, h = u % a.Hkv;
  __syncthreads();
  for (int idx = tid; idx < G * kHeadDim; idx += kAttnThreads) {
    const int g = idx / kHeadDim, d = idx % kHeadDim;
    float M = sm.m[0][g];
#pragma unroll
    for (int w = 1; w < kAttnWaves; ++w) M = fmaxf(M, sm.m[w][g]);
    const float Ms = M == -INFINITY ? 0.f : M;
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) {
      const float sc = exp2f(sm.m[w][g] - Ms);
      L += sm.l[w][g] * sc;
      A += sm.acc[w][g][d] * sc;
    }
    if (a.S == 1) {
      const size_t row = (size_t)b * a.Hq + (size_t)h * G + g;
      a.out[row * kHeadDim + d] = A / L;
      if (a.lse != nullptr && d == 0) a.lse[row] = (M + log2f(L)) * kLn2;
    } else {
      const size_t base = ((size_t)u * a.S + split) * G + g;
      a.part_acc[base * kHeadDim + d] = A;
      if (d == 0) {
        a.part_ml[base * 2] = M;
        a.part_ml[base * 2 + 1] = L;
      }
    }
  }
  if (a.S == 1 || !a.fuse_merge) return;
  __threadfence();                                   // partials visible device-wide before the ticket
  __syncthreads();
  if (tid == 0) {
    const int t = atomicAdd(&a.ticket[u], 1);
    sm.is_last = (t == a.S - 1) ? 1 : 0;
    if (t == a.S - 1) a.ticket[u] = 0;               // ready for the next launch
  }
  __syncthreads();
  if (!sm.is_last) return;
  __threadfence();
  merge_splits<G>(a, u);
}

template <int G>
__global__ __launch_bounds__(kAttnThreads) void combine_kernel(AttnArgs a) {
  merge_splits<G>(a, blockIdx.x + a.u0);
}

// ---------------------------------------------------------------------------------------------
// MFMA kernel (page size a multiple of 16, tile-layout slots)
// ---------------------------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

template <bool BF16>
__device__ __forceinline__ f32x4 mfma_qk(const uint4& kfrag, const uint4& qfrag, f32x4 c) {
  if (BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kfrag), __builtin_bit_cast(bf16x8, qfrag), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, kfrag), __builtin_bit_cast(f16x8, qfrag), c, 0, 0, 0);
}

template <bool BF16>
__device__ __forceinline__ f32x4 mfma_pv(const uint2& vfrag, const uint2& pfrag, f32x4 c) {
  if (BF16)
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, vfrag), __builtin_bit_cast(s16x4, pfrag), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, vfrag), __builtin_bit_cast(f16x4, pfrag), c, 0, 0, 0);
}

// Block (split, u): wave w takes 16-token tiles first + w, first + w + 4, ... of the split's pages.
// Per tile: 4 loads give the K operand (lane (i, g) = token i, dims 32c+8g..+7), 4 loads the V^T
// operands; S^T[token][head] = sum_c mfma(K_c, Q^T_c); the C tile of lane (j, g) holds head j,
// tokens 4g..4g+3, which is exactly the B operand of O^T[dim][head] += V^T[dim][token] P^T[token][head].
// Heads sit in the 16 MFMA columns; columns >= G carry zeros and are never read.
// For bf16 the probabilities are split into a high and a low bf16 part (two MFMAs) so that P
// keeps 16 bits of mantissa; fp16 P has 11 bits and needs one.
template <bool BF16, int G>
__global__ __launch_bounds__(kAttnThreads) void attend_mfma_kernel(AttnArgs a) {
  __shared__ AttnSmem<G> sm;
  __shared__ int32_t sh_page[kAttnIdxCap], sh_slot[kAttnIdxCap];
  const int split = blockIdx.x, u = blockIdx.y + a.u0;
  const int b = u / a.Hkv, h = u % a.Hkv;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int j = lane & 15, g = lane >> 4;

  // Q^T operand: lane (j, g) holds Q[head j][32c + 8g .. +7] for c = 0..3 (zeros for j >= G)
  uint4 qfrag[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) qfrag[c] = make_uint4(0u, 0u, 0u, 0u);
  if (j < G) {
    const uint16_t* qrow = a.q + ((size_t)b * a.Hq + (size_t)h * G + j) * kHeadDim + 8 * g;
#pragma unroll
    for (int c = 0; c < 4; ++c) qfrag[c] = *reinterpret_cast<const uint4*>(qrow + 32 * c);
  }

  f32x4 o[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  const int seq = a.seq_len[b];
  const int tiles_per_page = a.P >> 4;
  const int first = split * a.per_split;
  const int last = (first + a.per_split) < a.k ? (first + a.per_split) : a.k;
  const int n_tiles = (last - first) * tiles_per_page;
  const int32_t* sel = a.sel_pages + (size_t)u * a.k;
  const int32_t* slots = a.sel_slots + (size_t)u * a.k;
  const char* pool_u = a.pool + (size_t)u * a.Cmax * a.page_bytes;

  // the split's (page, slot) entries go to LDS once, so that issuing a tile's loads never waits on
  // a global index load
  const int n_entries = last - first;
  const bool idx_in_lds = n_entries <= kAttnIdxCap;
  if (idx_in_lds) {
    for (int i = tid; i < n_entries; i += kAttnThreads) {
      sh_page[i] = sel[first + i];
      sh_slot[i] = slots[first + i];
    }
  }
  __syncthreads();

  // software pipeline: three tile buffers rotate, so the operands of the next two tiles of this
  // wave (16 KiB) are in flight while one tile is computed
  struct Tile { uint4 k[4], v[4]; int ntok; };
  auto issue = [&](Tile& tl, int t) {
    tl.ntok = 0;
    if (t >= n_tiles) return;
    const int e = t / tiles_per_page, tile = t % tiles_per_page;
    const int page = __builtin_amdgcn_readfirstlane(idx_in_lds ? sh_page[e] : sel[first + e]);
    const int slot = __builtin_amdgcn_readfirstlane(idx_in_lds ? sh_slot[e] : slots[first + e]);
    if (page < 0 || slot < 0 || slot >= a.Cmax) return;
    int ntok = seq - page * a.P - tile * 16;
    ntok = ntok < 16 ? ntok : 16;
    if (ntok <= 0) return;
    tl.ntok = ntok;
    const uint4* tb = reinterpret_cast<const uint4*>(pool_u + (size_t)slot * a.page_bytes + (size_t)tile * kTileBytes) + lane;
#pragma unroll
    for (int c = 0; c < 4; ++c) tl.k[c] = load_stream16(tb + c * 64);
#pragma unroll
    for (int c = 0; c < 4; ++c) tl.v[c] = load_stream16(tb + 256 + c * 64);
  };
  auto compute = [&](const Tile& tl) {
    const int ntok = tl.ntok;
    if (ntok == 0) return;
    f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c) s = mfma_qk<BF16>(tl.k[c], qfrag[c], s);
    float x[4];
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[e] = (4 * g + e) < ntok ? s[e] * a.scale_log2 : -INFINITY;
      mx = fmaxf(mx, x[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float m_new = fmaxf(m, mx);                // finite: token 0 of the tile is valid
    if (__any(m_new > m)) {
      const float alpha = exp2f(m - m_new);
      l *= alpha;
#pragma unroll
      for (int c = 0; c < 8; ++c) o[c] *= alpha;
      m = m_new;
    }
    float p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      p[e] = exp2f(x[e] - m);
      l += p[e];
    }
    if (BF16) {
      const bf16x4 hi = {(__bf16)p[0], (__bf16)p[1], (__bf16)p[2], (__bf16)p[3]};
      const bf16x4 lo = {(__bf16)(p[0] - (float)hi[0]), (__bf16)(p[1] - (float)hi[1]), (__bf16)(p[2] - (float)hi[2]),
                         (__bf16)(p[3] - (float)hi[3])};
      const uint2 ph = __builtin_bit_cast(uint2, hi), pl = __builtin_bit_cast(uint2, lo);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint2 v0 = make_uint2(tl.v[c].x, tl.v[c].y), v1 = make_uint2(tl.v[c].z, tl.v[c].w);
        o[2 * c] = mfma_pv<true>(v0, ph, o[2 * c]);
        o[2 * c + 1] = mfma_pv<true>(v1, ph, o[2 * c + 1]);
        o[2 * c] = mfma_pv<true>(v0, pl, o[2 * c]);
        o[2 * c + 1] = mfma_pv<true>(v1, pl, o[2 * c + 1]);
      }
    } else {
      const f16x4 hp = {(_Float16)p[0], (_Float16)p[1], (_Float16)p[2], (_Float16)p[3]};
      const uint2 ph = __builtin_bit_cast(uint2, hp);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint2 v0 = make_uint2(tl.v[c].x, tl.v[c].y), v1 = make_uint2(tl.v[c].z, tl.v[c].w);
        o[2 * c] = mfma_pv<false>(v0, ph, o[2 * c]);
        o[2 * c + 1] = mfma_pv<false>(v1, ph, o[2 * c + 1]);
      }
    }
  };
  Tile ta, tb2, tc;
  issue(ta, w);
  issue(tb2, w + kAttnWaves);
  for (int t = w; t < n_tiles; t += 3 * kAttnWaves) {
    issue(tc, t + 2 * kAttnWaves);
    compute(ta);
    issue(ta, t + 3 * kAttnWaves);
    compute(tb2);
    issue(tb2, t + 4 * kAttnWaves);
    compute(tc);
  }

  // per-lane sums cover tokens 4g..4g+3 of every tile: add the four lane groups of a head
  l += __shfl_xor(l, 16, kWave);
  l += __shfl_xor(l, 32, kWave);
  if (j < G) {
    // O^T C tiles: lane (j, g) register e of tile c holds dim 16c + 4g + e of head j
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) sm.acc[w][j][16 * c + 4 * g + e] = o[c][e];
    if (g == 0) { sm.m[w][j] = m; sm.l[w][j] = l; }
  }
  finish_split<G>(a, sm, u, split);
}

// ---------------------------------------------------------------------------------------------
// VALU kernel (any page size, natural slots)
// ---------------------------------------------------------------------------------------------
// Block (split, u): 4 waves, wave w takes selected entries first + w, first + w + 4, ...
// A wave load covers 4 token rows: lane (r, c) = (lane / 16, lane % 16) holds dims 8c..8c+7 of
// token 4j + r of a 16-token tile.  Each 16-lane row keeps its own running (max, sum, acc) for the
// G query heads, so nothing crosses rows inside the loop; rows and waves are merged at the end.
template <bool BF16, int G>
__global__ __launch_bounds__(kAttnThreads) void attend_valu_kernel(AttnArgs a) {
  __shared__ AttnSmem<G> sm;
  const int split = blockIdx.x, u = blockIdx.y + a.u0;
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
      for (int jj = 0; jj < 4; ++jj) {
        int tok = t0 + 4 * jj + r;
        tok = tok < ntok ? tok : ntok - 1;
        kraw[jj] = *reinterpret_cast<const uint4*>(kbase + (size_t)tok * kRowBytes);
        vraw[jj] = *reinterpret_cast<const uint4*>(vbase + (size_t)tok * kRowBytes);
      }
      float x[4][G];
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        float kf[8];
        cvt8<BF16>(kraw[jj], kf);
        const bool valid = (t0 + 4 * jj + r) < ntok;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float s = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) s = fmaf(qf[g][e], kf[e], s);
          s = row16_allreduce_sum(s);
          x[jj][g] = valid ? s * a.scale_log2 : -INFINITY;
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
        for (int jj = 0; jj < 4; ++jj) {
          p[jj][g] = exp2f(x[jj][g] - m_safe);
          ps += p[jj][g];
        }
        l[g] = l[g] * alpha + ps;
        m[g] = m_new;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] *= alpha;
      }
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        float vf[8];
        cvt8<BF16>(vraw[jj], vf);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(p[jj][g], vf[e], acc[g][e]);
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
      for (int e = 0; e < 8; ++e) sm.acc[w][g][c * 8 + e] = acc[g][e];
      if (c == 0) { sm.m[w][g] = m[g]; sm.l[w][g] = l[g]; }
    }
  }
  finish_split<G>(a, sm, u, split);
}

template <bool BF16, int G>
static void launch_attend(bool tiled, const AttnArgs& a, dim3 grid, hipStream_t s, hipEvent_t between) {
  if (tiled)
    hipLaunchKernelGGL((attend_mfma_kernel<BF16, G>), grid, dim3(kAttnThreads), 0, s, a);
  else
    hipLaunchKernelGGL((attend_valu_kernel<BF16, G>), grid, dim3(kAttnThreads), 0, s, a);
  if (between != nullptr) (void)hipEventRecord(between, s);
  if (a.S > 1 && !a.fuse_merge)
    hipLaunchKernelGGL((combine_kernel<G>), dim3(grid.y), dim3(kAttnThreads), 0, s, a);
}

template <bool BF16>
static bool dispatch_group(int G, bool tiled, const AttnArgs& a, dim3 grid, hipStream_t s, hipEvent_t between) {
  switch (G) {
    case 1: launch_attend<BF16, 1>(tiled, a, grid, s, between); return true;
    case 2: launch_attend<BF16, 2>(tiled, a, grid, s, between); return true;
    case 3: launch_attend<BF16, 3>(tiled, a, grid, s, between); return true;
    case 4: launch_attend<BF16, 4>(tiled, a, grid, s, between); return true;
    case 5: launch_attend<BF16, 5>(tiled, a, grid, s, between); return true;
    case 6: launch_attend<BF16, 6>(tiled, a, grid, s, between); return true;
    case 7: launch_attend<BF16, 7>(tiled, a, grid, s, between); return true;
    case 8: launch_attend<BF16, 8>(tiled, a, grid, s, between); return true;
    default: return false;
  }
}

}  // namespace kvd

hipError_t kvd_launch_attend(kvd_ctx* c, int layer, const void* q, const int32_t* sel_pages,
                             const int32_t* sel_slots, float* out, float* lse, int u0, int u1, hipStream_t s,
                             hipEvent_t between) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  AttnArgs a;
  a.u0 = u0;
  a.q = reinterpret_cast<const uint16_t*>(q);
  a.pool = c->pool + (size_t)layer * c->U * c->Cmax * c->page_bytes;
  a.sel_pages = sel_pages;
  a.sel_slots = sel_slots;
  a.seq_len = c->d_seq_len;
  a.part_acc = c->d_part_acc;
  a.part_ml = c->d_part_ml;
  a.ticket = c->d_attn_ticket;
  a.out = out;
  a.lse = lse;
  a.k = c->k; a.P = c->P; a.Cmax = c->Cmax; a.Hq = c->Hq; a.Hkv = c->Hkv; a.S = c->S;
  a.per_split = (c->k + c->S - 1) / c->S;
  a.fuse_merge = c->fuse_merge;
  a.page_bytes = (unsigned)c->page_bytes;
  a.scale_log2 = c->scale * kLog2e;
  dim3 grid(c->S, u1 - u0);
  const bool ok = c->bf16 ? dispatch_group<true>(c->G, c->tiled != 0, a, grid, s, between)
                          : dispatch_group<false>(c->G, c->tiled != 0, a, grid, s, between);
  if (!ok) return hipErrorInvalidValue;
  return hipGetLastError();
}
