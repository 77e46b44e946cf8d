// Stage 3 of the decode step: GQA decode attention over the selected pages only (System
// Overview: attention runs over the union of resident and newly fetched entries).  See
// kvd_attn_body.h for the split-K frame.
//
// Two kernels share that frame:
//  * attend_mfma_kernel — pages whose size is a multiple of 16 tokens are kept in the slot pool in
//    an operand-ready tile layout (see kvd_tile_layout.h), so that every wave load is 1 KiB
//    contiguous and lands directly in MFMA operand registers: S^T = K Q^T with 16x16x32 MFMAs,
//    O^T += V^T P^T with 16x16x16 MFMAs whose B operand is the softmaxed C tile of the first.
//    Pages of 4 or 8 tokens take the same kernel over the packed layout: 16 / P pages per tile.
//  * attend_valu_kernel — any page size, natural [token][dim] slots, fp32 VALU arithmetic.
#include <math.h>

#include <mutex>

#include "kvd_attn_body.h"
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_tile_layout.h"

// Scratch of kvd_sparse_decode_attn_noalloc: the arrival tickets of the units, then the split
// partials (max and sum per query head, then the accumulators).  Every GPU the library runs on
// holds its own copy of this array from the moment the code is loaded until the process ends.
constexpr size_t kNoAllocScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

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
template <bool BF16, int G, bool PACKED>
__global__ __launch_bounds__(kAttnMfmaThreads, 2) void attend_mfma_kernel(AttnArgs a) {
  __shared__ AttnSmem<G, kAttnMfmaThreads / kWave> sm;
  attend_mfma_body<BF16, G, kAttnMfmaThreads, false, false, PACKED>(a, sm, blockIdx.y + a.u0, blockIdx.x);
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
static void launch_attend(int layout, const AttnArgs& a, dim3 grid, hipStream_t s, hipEvent_t between) {
  if (layout == kLayoutPacked)
    hipLaunchKernelGGL((attend_mfma_kernel<BF16, G, true>), grid, dim3(kAttnMfmaThreads), 0, s, a);
  else if (layout == kLayoutTiles)
    hipLaunchKernelGGL((attend_mfma_kernel<BF16, G, false>), grid, dim3(kAttnMfmaThreads), 0, s, a);
  else
    hipLaunchKernelGGL((attend_valu_kernel<BF16, G>), grid, dim3(kAttnThreads), 0, s, a);
  if (between != nullptr) (void)hipEventRecord(between, s);   // no kernel follows when the merge is fused
  if (a.S > 1 && !a.fuse_merge)
    hipLaunchKernelGGL((combine_kernel<G>), dim3(grid.y), dim3(kAttnThreads), 0, s, a);
}

template <bool BF16>
static bool dispatch_group(int G, int layout, const AttnArgs& a, dim3 grid, hipStream_t s, hipEvent_t between) {
  switch (G) {
    case 1: launch_attend<BF16, 1>(layout, a, grid, s, between); return true;
    case 2: launch_attend<BF16, 2>(layout, a, grid, s, between); return true;
    case 3: launch_attend<BF16, 3>(layout, a, grid, s, between); return true;
    case 4: launch_attend<BF16, 4>(layout, a, grid, s, between); return true;
    case 5: launch_attend<BF16, 5>(layout, a, grid, s, between); return true;
    case 6: launch_attend<BF16, 6>(layout, a, grid, s, between); return true;
    case 7: launch_attend<BF16, 7>(layout, a, grid, s, between); return true;
    case 8: launch_attend<BF16, 8>(layout, a, grid, s, between); return true;
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
  const bool ok = c->bf16 ? dispatch_group<true>(c->G, c->tiled, a, grid, s, between)
                          : dispatch_group<false>(c->G, c->tiled, a, grid, s, between);
  if (!ok) return hipErrorInvalidValue;
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------------
// The attention stage for callers that cannot allocate
// ---------------------------------------------------------------------------------------------
namespace {

constexpr int kMaxDevices = 64;
std::mutex g_noalloc_mutex;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU (the array's name is only a host-side handle)
int g_scratch_cus[kMaxDevices];

// Device address of this GPU's copy of `scratch` and its number of compute units, looked up once
// per device with that device current.
hipError_t noalloc_device_state(void** ptr, int* cus) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_noalloc_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    int n = 0;
    e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    g_scratch_cus[dev] = n > 0 ? n : 256;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  *cus = g_scratch_cus[dev];
  return hipSuccess;
}

size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

extern "C" int kvd_sparse_decode_attn_noalloc(const void* q, const void* slot_pool, const int32_t* sel_pages,
                                              const int32_t* sel_slots, const int32_t* seq_len, float* out, float* lse,
                                              int32_t batch, int32_t n_q_heads, int32_t n_kv_heads, int32_t page_size,
                                              int32_t topk_pages, int32_t capacity_max, int32_t kv_dtype,
                                              float softmax_scale, int32_t attn_splits, void* stream) {
  using namespace kvd;
  if (!q || !slot_pool || !sel_pages || !sel_slots || !seq_len || !out) return KVD_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(q) & 15u) || (reinterpret_cast<uintptr_t>(slot_pool) & 15u)) return KVD_ERR_ARG;
  if (kv_dtype != KVD_F16 && kv_dtype != KVD_BF16) return KVD_ERR_DTYPE;
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0) return KVD_ERR_SHAPE;
  const int G = n_q_heads / n_kv_heads;
  if (G > KVD_MAX_GROUP) return KVD_ERR_SHAPE;
  if (page_size < 1 || page_size > KVD_MAX_PAGE) return KVD_ERR_SHAPE;
  if (topk_pages < 1 || topk_pages > KVD_MAX_TOPK) return KVD_ERR_SHAPE;
  if (capacity_max < 1 || capacity_max > KVD_MAX_CAPACITY) return KVD_ERR_SHAPE;
  if ((long long)batch * n_kv_heads > 65535) return KVD_ERR_SHAPE;
  if (attn_splits < 0 || attn_splits > KVD_MAX_SPLITS) return KVD_ERR_SHAPE;
  if (!(softmax_scale >= 0.f) || isinf(softmax_scale)) return KVD_ERR_ARG;
  void* base = nullptr;
  int cus = 0;
  // (the number of compute units is only needed to choose the splits: sizes that cannot fit
  // whatever the device are refused before any device is touched)
  if (attn_splits == 0 && noalloc_device_state(&base, &cus) != hipSuccess) {
    (void)hipGetLastError();
    return KVD_ERR_HIP;
  }
  const int U = batch * n_kv_heads;
  const int layout = slot_layout_of(page_size);
  const bool tiled = layout != kLayoutNatural;
  // split-K factor: the rule of kvd_create
  int S = attn_splits;
  if (S == 0) {
    const int tiles = layout == kLayoutPacked ? (topk_pages * page_size + 15) / 16 : topk_pages * ((page_size + 15) / 16);
    if (tiled) {
      S = (cus + U / 2) / U;
      if (S > tiles / 16) S = tiles / 16;
    } else {
      S = (512 + U / 2) / U;
      if (S > (tiles + 7) / 8) S = (tiles + 7) / 8;
    }
    if (S > KVD_MAX_SPLITS) S = KVD_MAX_SPLITS;
    if (S < 1) S = 1;
  }
  if (S > topk_pages) S = topk_pages;
  // the scratch array, cut into tickets [U], (max, sum) [U][S][G][2] and accumulators [U][S][G][D]
  const size_t rows = (size_t)U * S * G;
  const size_t off_ml = round256((size_t)U * sizeof(int32_t));
  const size_t off_acc = off_ml + round256(rows * 2 * sizeof(float));
  const size_t need = off_acc + rows * kHeadDim * sizeof(float);
  if (need > kNoAllocScratchBytes) return KVD_ERR_CAPACITY;
  if (base == nullptr && noalloc_device_state(&base, &cus) != hipSuccess) {
    (void)hipGetLastError();
    return KVD_ERR_HIP;
  }
  unsigned char* sp = static_cast<unsigned char*>(base);
  hipStream_t s = static_cast<hipStream_t>(stream);

  AttnArgs a;
  a.u0 = 0;
  a.q = reinterpret_cast<const uint16_t*>(q);
  a.pool = static_cast<const char*>(slot_pool);
  a.sel_pages = sel_pages;
  a.sel_slots = sel_slots;
  a.sel_entry = nullptr;
  a.error = nullptr;
  a.wait_limit = 0;
  a.seq_len = seq_len;
  a.ticket = reinterpret_cast<int32_t*>(sp);
  a.part_ml = reinterpret_cast<float*>(sp + off_ml);
  a.part_acc = reinterpret_cast<float*>(sp + off_acc);
  a.out = out;
  a.lse = lse;
  a.k = topk_pages; a.P = page_size; a.Cmax = capacity_max; a.Hq = n_q_heads; a.Hkv = n_kv_heads; a.G = G; a.S = S;
  a.per_split = (topk_pages + S - 1) / S;
  a.fuse_merge = 1;
  a.page_bytes = (unsigned)((size_t)2 * page_size * kHeadDim * 2);
  a.scale_log2 = (softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)kHeadDim)) * kLog2e;
  // the tickets must start at zero whatever an earlier call left there (a fill kernel, so that
  // the call can be captured into a HIP graph)
  if (S > 1 && kvd_launch_fill_i32(a.ticket, 0, (size_t)U, s) != hipSuccess) {
    (void)hipGetLastError();
    return KVD_ERR_HIP;
  }
  const dim3 grid(S, U);
  const bool ok = kv_dtype == KVD_BF16 ? dispatch_group<true>(G, layout, a, grid, s, nullptr)
                                       : dispatch_group<false>(G, layout, a, grid, s, nullptr);
  if (!ok) return KVD_ERR_SHAPE;
  if (hipGetLastError() != hipSuccess) return KVD_ERR_HIP;
  return KVD_OK;
}
