// Stage 3 of the decode step: GQA decode attention over the selected pages only (System
// Overview: attention runs over the union of resident and newly fetched entries).  See
// kvd_attn_body.h for the split-K frame.
//
// Two kernels share that frame:
//  * attend_mfma_kernel — pages whose size is a multiple of 16 tokens are kept in the slot pool in
//    an operand-ready tile layout (see kvd_tile_layout.h), so that every wave load is 1 KiB
//    contiguous and lands directly in MFMA operand registers: S^T = K Q^T with 16x16x32 MFMAs,
//    O^T += V^T P^T with 16x16x16 MFMAs whose B operand is the softmaxed C tile of the first.
//  * attend_valu_kernel — any page size, natural [token][dim] slots, fp32 VALU arithmetic.
#include "kvd_attn_body.h"
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_tile_layout.h"

namespace kvd {

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = kAttnThreads / kWave;

template <int G>
__global__ __launch_bounds__(kAttnThreads) void combine_kernel(AttnArgs a) {
  merge_splits<G, kAttnThreads, false>(a, blockIdx.x + a.u0);
}

// 512 threads and up to 256 registers per lane: one workgroup per CU, three tile buffers (24 KiB)
// in flight per wave; the grid is sized to about one workgroup per CU (see kvd_create).
constexpr int kAttnMfmaThreads = 512;
template <bool BF16, int G>
__global__ __launch_bounds__(kAttnMfmaThreads, 2) void attend_mfma_kernel(AttnArgs a) {
  __shared__ AttnSmem<G, kAttnMfmaThreads / kWave> sm;
  attend_mfma_body<BF16, G, kAttnMfmaThreads, false>(a, sm, blockIdx.y + a.u0, blockIdx.x);
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
  __shared__ AttnSmem<G, kAttnWaves> sm;
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
  finish_split<G, kAttnThreads>(a, sm, u, split);
}

template <bool BF16, int G>
static void launch_attend(bool tiled, const AttnArgs& a, dim3 grid, hipStream_t s, hipEvent_t between) {
  if (tiled)
    hipLaunchKernelGGL((attend_mfma_kernel<BF16, G>), grid, dim3(kAttnMfmaThreads), 0, s, a);
  else
    hipLaunchKernelGGL((attend_valu_kernel<BF16, G>), grid, dim3(kAttnThreads), 0, s, a);
  if (between != nullptr) (void)hipEventRecord(between, s);   // no kernel follows when the merge is fused
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

kvd::AttnArgs kvd_attn_args(kvd_ctx* c, int layer, const void* q, const int32_t* sel_pages, const int32_t* sel_slots,
                            float* out, float* lse, int u0) {
  using namespace kvd;
  AttnArgs a;
  a.u0 = u0;
  a.q = reinterpret_cast<const uint16_t*>(q);
  a.pool = c->pool + (size_t)layer * c->U * c->Cmax * c->page_bytes;
  a.sel_pages = sel_pages;
  a.sel_slots = sel_slots;
  a.sel_entry = nullptr;                               // (only the one-launch step hands the selection over in entries)
  a.error = c->error_dev;
  a.wait_limit = c->wait_limit_ticks;
  a.seq_len = c->d_seq_len;
  a.part_acc = c->d_part_acc;
  a.part_ml = c->d_part_ml;
  a.ticket = c->d_attn_ticket;
  a.out = out;
  a.lse = lse;
  a.k = c->k; a.P = c->P; a.Cmax = c->Cmax; a.Hq = c->Hq; a.Hkv = c->Hkv; a.G = c->G; a.S = c->S;
  a.per_split = (c->k + c->S - 1) / c->S;
  a.fuse_merge = c->fuse_merge;
  a.page_bytes = (unsigned)c->page_bytes;
  a.scale_log2 = c->scale * kLog2e;
  return a;
}

hipError_t kvd_launch_attend(kvd_ctx* c, int layer, const void* q, const int32_t* sel_pages,
                             const int32_t* sel_slots, float* out, float* lse, int u0, int u1, hipStream_t s,
                             hipEvent_t between) {
  using namespace kvd;
  if (u1 <= u0) return hipSuccess;
  const AttnArgs a = kvd_attn_args(c, layer, q, sel_pages, sel_slots, out, lse, u0);
  dim3 grid(c->S, u1 - u0);
  const bool ok = c->bf16 ? dispatch_group<true>(c->G, c->tiled != 0, a, grid, s, between)
                          : dispatch_group<false>(c->G, c->tiled != 0, a, grid, s, between);
  if (!ok) return hipErrorInvalidValue;
  return hipGetLastError();
}
