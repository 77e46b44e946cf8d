// Device-side helpers shared by the kvd kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvd {

typedef unsigned long long u64;
typedef uint32_t u32;

constexpr int kWave = 64;
constexpr int kHeadDim = 128;
constexpr int kRowBytes = kHeadDim * 2;   // one token's K (or V) row: 128 x 2 bytes
constexpr int kRadixBits = 11;
constexpr int kRadixBins = 1 << kRadixBits;

__device__ __forceinline__ float as_f32(u32 x) { return __uint_as_float(x); }
__device__ __forceinline__ u32 as_u32(float x) { return __float_as_uint(x); }

// ---- streaming 16-byte load: data that is read once per launch is fetched with the non-temporal
// hint so that it does not displace reusable lines from the caches
typedef u32 u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- data handed from one workgroup to another inside one launch ------------------------------
// Workgroups of a launch may run on different XCDs, each with its own L2.  Values that one
// workgroup produces and another consumes in the same launch are therefore moved with
// device-scope accesses (written through to, and read from, the memory side), and a flag is
// raised only after the producer's stores have been acknowledged.
template <class T>
__device__ __forceinline__ T load_agent(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T>
__device__ __forceinline__ void store_agent(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// All memory operations this wave has issued are complete (loads returned, stores acknowledged).
__device__ __forceinline__ void wave_drain_memory() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
}

// Thread 0 polls *flag until it equals `want` (device-scope loads, sleeping between polls) or
// until `limit` ticks of the 100 MHz wall clock have passed; the verdict is shared through
// *lds_ok.  Returns false on a time-out.  Contains a barrier: call from all threads.
__device__ __forceinline__ bool block_wait_equal(const int32_t* flag, int32_t want, long long limit, int* lds_ok) {
  if (threadIdx.x == 0) {
    int ok = 1;
    if (load_agent(flag) != want) {
      const long long t0 = wall_clock64();
      for (;;) {
        __builtin_amdgcn_s_sleep(8);
        if (load_agent(flag) == want) break;
        if (wall_clock64() - t0 > limit) { ok = 0; break; }
      }
    }
    *lds_ok = ok;
  }
  __syncthreads();
  return *lds_ok != 0;
}

// ---- 16-bit -> fp32, eight elements of one 16-byte load -------------------------------------
template <bool BF16>
__device__ __forceinline__ void cvt8(const uint4& raw, float (&f)[8]) {
  const u32 w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (BF16) {
      f[2 * i] = as_f32(w[i] << 16);
      f[2 * i + 1] = as_f32(w[i] & 0xffff0000u);
    } else {
      typedef _Float16 h2 __attribute__((ext_vector_type(2)));
      h2 v = __builtin_bit_cast(h2, w[i]);
      f[2 * i] = (float)v.x;
      f[2 * i + 1] = (float)v.y;
    }
  }
}

// ---- cross-lane ------------------------------------------------------------------------------
// Sum over the 16 lanes of a DPP row (lanes 16r .. 16r+15); every lane gets the total.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_allreduce_sum(float v) {
  v += dpp_mov<0x128>(v);   // row_ror:8
  v += dpp_mov<0x124>(v);   // row_ror:4
  v += dpp_mov<0x122>(v);   // row_ror:2
  v += dpp_mov<0x121>(v);   // row_ror:1
  return v;
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP moves only: log-step shifts inside
// each row of 16 lanes (lanes shifted in from outside the row read 0), then the last lane of
// row 0 / row 2 is added to row 1 / row 3, then lane 31 to rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_get(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, true);
}
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_get<0x111, 0xf>(v);   // row_shr:1
  v += dpp_get<0x112, 0xf>(v);   // row_shr:2
  v += dpp_get<0x114, 0xf>(v);   // row_shr:4
  v += dpp_get<0x118, 0xf>(v);   // row_shr:8
  v += dpp_get<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_get<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}

// Exclusive prefix sum of one int per thread over the block; `total` gets the block sum.
// `smem` holds at least NT/64 + 1 ints.  Two barriers inside; safe to call back to back.
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int v, int* smem, int& total) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int inc = wave_inclusive_scan(v);
  __syncthreads();                       // previous users of smem are done
  if (lane == kWave - 1) smem[w] = inc;
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const int t = smem[i];
    if (i < w) base += t;
    tot += t;
  }
  total = tot;
  return base + inc - v;
}

// min / max / sum over the 64 lanes with DPP rotations inside the rows of 16 and two cross-row
// exchanges; every lane gets the result
__device__ __forceinline__ float wave_allreduce_min(float v) {
  v = fminf(v, dpp_mov<0x128>(v));
  v = fminf(v, dpp_mov<0x124>(v));
  v = fminf(v, dpp_mov<0x122>(v));
  v = fminf(v, dpp_mov<0x121>(v));
  v = fminf(v, __shfl_xor(v, 16, kWave));
  return fminf(v, __shfl_xor(v, 32, kWave));
}
__device__ __forceinline__ float wave_allreduce_max(float v) {
  v = fmaxf(v, dpp_mov<0x128>(v));
  v = fmaxf(v, dpp_mov<0x124>(v));
  v = fmaxf(v, dpp_mov<0x122>(v));
  v = fmaxf(v, dpp_mov<0x121>(v));
  v = fmaxf(v, __shfl_xor(v, 16, kWave));
  return fmaxf(v, __shfl_xor(v, 32, kWave));
}

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int m) {
  u32 lo = (u32)v, hi = (u32)(v >> 32);
  lo = __shfl_xor((int)lo, m, kWave);
  hi = __shfl_xor((int)hi, m, kWave);
  return ((u64)hi << 32) | lo;
}

// ---- exact k-th smallest of distinct 64-bit keys, one block ----------------------------------
struct SelectSmem {
  int scan[32];
  u64 red_min[16];
  u64 red_max[16];
  u64 lo, hi;
  int need;
  int bin, below;
};

// `hist` is an LDS array of kRadixBins counters.
// keyfn(i, key) -> bool valid, for i in [0, n).  Keys must be distinct.  `need` is 1-based and
// at most the number of valid items.  Returns the need-th smallest key.  All threads of the block
// must call it with the same arguments.  Radix refinement: at most ceil(64/11) counting passes,
// each narrowing the inclusive key range [lo, hi] to one of 2048 equal sub-ranges.
template <int NT, class KeyFn>
__device__ u64 block_kth_smallest(KeyFn keyfn, int n, int need, SelectSmem& sm, u32* hist) {
  constexpr int NW = NT / kWave;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  u64 mn = ~0ull, mx = 0ull;
  for (int i = tid; i < n; i += NT) {
    u64 key;
    if (keyfn(i, key)) {
      mn = key < mn ? key : mn;
      mx = key > mx ? key : mx;
    }
  }
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    const u64 a = shfl_xor_u64(mn, m), b = shfl_xor_u64(mx, m);
    mn = a < mn ? a : mn;
    mx = b > mx ? b : mx;
  }
  __syncthreads();
  if (lane == 0) { sm.red_min[w] = mn; sm.red_max[w] = mx; }
  __syncthreads();
  if (tid == 0) {
    u64 a = sm.red_min[0], b = sm.red_max[0];
    for (int i = 1; i < NW; ++i) {
      a = sm.red_min[i] < a ? sm.red_min[i] : a;
      b = sm.red_max[i] > b ? sm.red_max[i] : b;
    }
    sm.lo = a; sm.hi = b; sm.need = need;
  }
  __syncthreads();
  for (;;) {
    const u64 lo = sm.lo, hi = sm.hi;
    const int want = sm.need;
    if (lo == hi) return lo;
    const u64 width = hi - lo;
    const int bits = 64 - __clzll((long long)width);
    const int shift = bits > kRadixBits ? bits - kRadixBits : 0;
    for (int i = tid; i < kRadixBins; i += NT) hist[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += NT) {
      u64 key;
      if (keyfn(i, key) && key >= lo && key <= hi) atomicAdd(&hist[(u32)((key - lo) >> shift)], 1u);
    }
    __syncthreads();
    constexpr int BPT = kRadixBins / NT;           // consecutive bins per thread
    int local = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) local += (int)hist[tid * BPT + j];
    int total;
    int ex = block_exclusive_scan<NT>(local, sm.scan, total);
    if (ex < want && want <= ex + local) {         // exactly one thread
      int b = tid * BPT;
      for (int j = 0; j < BPT; ++j, ++b) {
        const int c = (int)hist[b];
        if (want <= ex + c) break;
        ex += c;
      }
      sm.bin = b; sm.below = ex;
    }
    __syncthreads();
    const u64 nlo = lo + ((u64)sm.bin << shift);
    const u64 span = shift == 0 ? 0ull : ((1ull << shift) - 1ull);
    const u64 nhi = (hi - nlo) < span ? hi : nlo + span;
    const int nneed = want - sm.below;
    __syncthreads();                                // everyone has read sm.* of this pass
    if (shift == 0) return nlo;
    if (tid == 0) { sm.lo = nlo; sm.hi = nhi; sm.need = nneed; }
    __syncthreads();
  }
}

// ---- fp64 -> fp16 / bf16 with one round-to-nearest-even ----------------------------------------
template <bool BF16>
__device__ __forceinline__ uint16_t f64_to_kv(double x) {
  constexpr int MB = BF16 ? 7 : 10;                // stored mantissa bits
  constexpr int EB = BF16 ? 8 : 5;
  constexpr int BIAS = (1 << (EB - 1)) - 1;
  constexpr int EMIN = 1 - BIAS;
  const u64 b = (u64)__double_as_longlong(x);
  const u32 sign = (u32)(b >> 63) << 15;
  const int ef = (int)((b >> 52) & 0x7ff);
  const u64 man = b & ((1ull << 52) - 1ull);
  const u32 exp_all = ((1u << EB) - 1u) << MB;
  if (ef == 0x7ff) return (uint16_t)(sign | exp_all | (man ? (1u << (MB - 1)) : 0u));
  if (ef == 0) return (uint16_t)sign;              // fp64 zero / subnormal: far below the target range
  int e = ef - 1023;
  const u64 full = man | (1ull << 52);
  int shift = 52 - MB;
  if (e < EMIN) shift += EMIN - e;
  if (shift > 54) return (uint16_t)sign;
  u64 q = full >> shift;
  const u64 rem = full & ((1ull << shift) - 1ull);
  const u64 half = 1ull << (shift - 1);
  if (rem > half || (rem == half && (q & 1ull))) ++q;
  if (e >= EMIN) {
    if (q == (1ull << (MB + 1))) { q >>= 1; ++e; }
    if (e > BIAS) return (uint16_t)(sign | exp_all);
    return (uint16_t)(sign | ((u32)(e + BIAS) << MB) | ((u32)q & ((1u << MB) - 1u)));
  }
  return (uint16_t)(sign | (u32)q);                // subnormal (or rounded up into the smallest normal)
}

}  // namespace kvd
