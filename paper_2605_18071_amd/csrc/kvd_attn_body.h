// GQA decode attention over the selected pages of one unit by one workgroup (System Overview:
// attention runs over the union of resident and newly fetched entries).  The selected pages of a
// unit are split over several workgroups (split-K); each streams its K/V pages from the slot pool
// once and keeps an fp32 online softmax per query head; the split partials are merged by
// log-sum-exp, either by the last workgroup of the unit to finish or by a second kernel.
// Shared by the stand-alone attention kernels and the single-launch layer-step kernel.
#pragma once
#include "kvd_device.h"
#include "kvd_internal.h"
#include "kvd_tile_layout.h"

namespace kvd {

constexpr int kAttnIdxCap = 512;          // (page, slot) entries of a split kept in LDS
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
  const uint16_t* q;         // [B][Hq][D]
  const char* pool;          // [U][Cmax] slots of the layer
  const int32_t* sel_pages;  // [U][k]
  const int32_t* sel_slots;  // [U][k]
  u64* sel_entry;            // [U][k]: what a HANDOFF caller reads instead of the two (see pack_sel_entry); cleared after use
  int32_t* error;            // host-visible word, raised when the wait for the entries runs out
  long long wait_limit;      // bound of that wait in ticks of the 100 MHz wall clock
  const int32_t* seq_len;    // [B]
  float* part_acc;           // [U][S][G][D]
  float* part_ml;            // [U][S][G][2]
  int32_t* ticket;           // [U], zero between launches
  float* out;                // [B][Hq][D]
  float* lse;                // [B][Hq] or null
  int k, P, Cmax, Hq, Hkv, G, S, per_split, fuse_merge, u0;
  unsigned page_bytes;
  float scale_log2;          // softmax scale * log2(e)
};

// GMAX query heads per KV head at most, NW waves per workgroup
template <int GMAX, int NW>
struct AttnSmem {
  float acc[NW][GMAX][kHeadDim];
  float m[NW][GMAX];
  float l[NW][GMAX];
  int32_t page[kAttnIdxCap], slot[kAttnIdxCap];
  uint4 qf[4][kWave];                      // Q^T operand fragments, when they are not kept in registers
  int is_last;
};

// GT > 0: the group size is the compile-time GT; GT == 0: it is a.G (at most KVD_MAX_GROUP).
template <int GT>
__device__ __forceinline__ int group_size(const AttnArgs& a) { return GT > 0 ? GT : a.G; }
template <int GT>
struct GroupMax { static constexpr int value = GT > 0 ? GT : KVD_MAX_GROUP; };

// Log-sum-exp merge of the S split partials of unit u into out / lse, by one workgroup of NT
// threads.  The partials are fetched in batches of 8 splits whose loads are all issued before any
// is used.  HANDOFF: the partials were written by other workgroups of the same launch.
template <int GT, int NT, bool HANDOFF>
__device__ __forceinline__ void merge_splits(const AttnArgs& a, int u) {
  const int G = group_size<GT>(a);
  const int tid = threadIdx.x;
  const int b = u / a.Hkv, h = u % a.Hkv;
  for (int idx = tid; idx < G * kHeadDim; idx += NT) {
    const int g = idx / kHeadDim, d = idx % kHeadDim;
    const float* ml = a.part_ml + ((size_t)u * a.S * G + g) * 2;
    const float* pa = a.part_acc + ((size_t)u * a.S * G + g) * kHeadDim + d;
    float M = -INFINITY, L = 0.f, A = 0.f;
    for (int s0 = 0; s0 < a.S; s0 += 8) {
      float mv[8], lv[8], av[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int s = (s0 + i) < a.S ? (s0 + i) : (a.S - 1);
        if (HANDOFF) {
          mv[i] = load_agent(ml + (size_t)s * G * 2);
          lv[i] = load_agent(ml + (size_t)s * G * 2 + 1);
          av[i] = load_agent(pa + (size_t)s * G * kHeadDim);
        } else {
          mv[i] = ml[(size_t)s * G * 2];
          lv[i] = ml[(size_t)s * G * 2 + 1];
          av[i] = pa[(size_t)s * G * kHeadDim];
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (s0 + i < a.S) {
          const float Mn = fmaxf(M, mv[i]);
          const float Ms = Mn == -INFINITY ? 0.f : Mn;
          const float so = exp2f(M - Ms), sn = exp2f(mv[i] - Ms);
          L = L * so + lv[i] * sn;
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

// Workgroup epilogue.  The waves have left their (max, sum, acc) in `sm`; merge them and write
// this split's partial.  With fuse_merge the partials travel with device-scope stores and the
// last split of the unit to arrive (a ticket counter) merges all S of them.
// Returns true in the workgroup that completed the unit's output (with a separate merge kernel:
// never).
template <int GT, int NT>
__device__ __forceinline__ bool finish_split(const AttnArgs& a, AttnSmem<GroupMax<GT>::value, NT / kWave>& sm, int u,
                                             int split) {
  constexpr int NW = NT / kWave;
  const int G = group_size<GT>(a);
  const int tid = threadIdx.x;
  const int b = u / a.Hkv, h = u % a.Hkv;
  const bool fused = a.fuse_merge != 0;
  __syncthreads();
  for (int idx = tid; idx < G * kHeadDim; idx += NT) {
    const int g = idx / kHeadDim, d = idx % kHeadDim;
    float M = sm.m[0][g];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, sm.m[w][g]);
    const float Ms = M == -INFINITY ? 0.f : M;
    float L = 0.f, A = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
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
      if (fused) {
        store_agent(&a.part_acc[base * kHeadDim + d], A);
        if (d == 0) {
          store_agent(&a.part_ml[base * 2], M);
          store_agent(&a.part_ml[base * 2 + 1], L);
        }
      } else {
        a.part_acc[base * kHeadDim + d] = A;
        if (d == 0) {
          a.part_ml[base * 2] = M;
          a.part_ml[base * 2 + 1] = L;
        }
      }
    }
  }
  if (a.S == 1) {
    // (a HANDOFF caller's entries were read into LDS before the first barrier: blank them for the next launch)
    if (a.sel_entry != nullptr)
      for (int i = tid; i < a.k; i += NT) store_agent(&a.sel_entry[(size_t)u * a.k + i], 0ull);
    return true;
  }
  if (!fused) return false;
  wave_drain_memory();                               // this wave's partials have been acknowledged
  __syncthreads();
  if (tid == 0) {
    const int t = __hip_atomic_fetch_add(&a.ticket[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm.is_last = (t == a.S - 1) ? 1 : 0;
    if (t == a.S - 1) store_agent(&a.ticket[u], 0);  // ready for the next launch
  }
  __syncthreads();
  if (!sm.is_last) return false;
  merge_splits<GT, NT, true>(a, u);
  // every split of the unit has read its entries: blank them for the next launch
  if (a.sel_entry != nullptr)
    for (int i = tid; i < a.k; i += NT) store_agent(&a.sel_entry[(size_t)u * a.k + i], 0ull);
  return true;
}

// ---------------------------------------------------------------------------------------------
// MFMA attention (page size a multiple of 16, tile-layout slots)
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

// Workgroup (split, u) of NT threads: wave w takes 16-token tiles first + w, first + w + NW, ... of
// the split's pages.  Per tile: 4 loads give the K operand (lane (i, g) = token i, dims
// 32c+8g..+7), 4 loads the V^T operands; S^T[token][head] = sum_c mfma(K_c, Q^T_c); the C tile of
// lane (j, g) holds head j, tokens 4g..4g+3, which is exactly the B operand of
// O^T[dim][head] += V^T[dim][token] P^T[token][head].  Heads sit in the 16 MFMA columns; columns
// >= G carry zeros and are never read.  For bf16 the probabilities are split into a high and a
// low bf16 part (two MFMAs) so that P keeps 16 bits of mantissa; fp16 P has 11 bits and needs one.
// HANDOFF: the selection was written by another workgroup of the same launch.
// LEAN: for 128 registers per lane (two workgroups of 8 waves per CU): two tile buffers instead of
// three and the Q^T fragments re-read from LDS for every tile.
// PACKED: pages of 4 or 8 tokens in the packed slot layout: a tile is made of 16 / P consecutive
// entries of the split, every lane fetching its 16-byte units from the slot of its own page, and
// every token of the tile is valid or not on its own (a page beyond the selection's end, a made-up
// page, the ragged last page of a sequence).
// Returns 1 in the workgroup that completed the unit's output, 0 in the others, -1 (from all
// threads, no output) when a HANDOFF wait ran out.  inputs_ready_tick (one thread passes it)
// receives the wall clock at which the split's entries were all there.
template <bool BF16, int GT, int NT, bool HANDOFF, bool LEAN = false, bool PACKED = false>
__device__ __forceinline__ int attend_mfma_body(const AttnArgs& a, AttnSmem<GroupMax<GT>::value, NT / kWave>& sm, int u,
                                                int split, long long* inputs_ready_tick = nullptr) {
  constexpr int NW = NT / kWave;
  const int G = group_size<GT>(a);
  const int b = u / a.Hkv, h = u % a.Hkv;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
  const int j = lane & 15, g = lane >> 4;

  // Q^T operand: lane (j, g) holds Q[head j][32c + 8g .. +7] for c = 0..3 (zeros for j >= G)
  uint4 qfrag[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) qfrag[c] = make_uint4(0u, 0u, 0u, 0u);
  if (!LEAN || w == 0) {
    if (j < G) {
      const uint16_t* qrow = a.q + ((size_t)b * a.Hq + (size_t)h * G + j) * kHeadDim + 8 * g;
#pragma unroll
      for (int c = 0; c < 4; ++c) qfrag[c] = *reinterpret_cast<const uint4*>(qrow + 32 * c);
    }
    if (LEAN) {
#pragma unroll
      for (int c = 0; c < 4; ++c) sm.qf[c][lane] = qfrag[c];
    }
  }

  f32x4 o[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) o[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m = -INFINITY, l = 0.f;

  const int seq = a.seq_len[b];
  const int tiles_per_page = a.P >> 4;                  // (PACKED: 0; pages_per_tile counts instead)
  const int pages_per_tile = PACKED ? 16 / a.P : 1;
  const int first = split * a.per_split;
  const int last = (first + a.per_split) < a.k ? (first + a.per_split) : a.k;
  const int n_tiles = PACKED ? (last - first + pages_per_tile - 1) / pages_per_tile : (last - first) * tiles_per_page;
  const int32_t* sel = a.sel_pages + (size_t)u * a.k;
  const int32_t* slots = a.sel_slots + (size_t)u * a.k;
  const char* pool_u = a.pool + (size_t)u * a.Cmax * a.page_bytes;

  // the split's (page, slot) entries go to LDS once, so that issuing a tile's loads never waits on
  // a global index load.  HANDOFF: they come from the unit's selection workgroup of the same launch,
  // one 64-bit word each, and a thread polls its word until it has been published (a word is
  // published when the page is in its slot); the wait is bounded and its verdict shared.
  const int n_entries = last - first;
  const bool idx_in_lds = HANDOFF || n_entries <= kAttnIdxCap;   // (HANDOFF callers keep splits within kAttnIdxCap)
  if (HANDOFF) {
    const u64* ent = a.sel_entry + (size_t)u * a.k + first;
    if (tid == 0) sm.is_last = 0;                      // (here: -1 once some thread's wait has run out)
    __syncthreads();
    int failed = 0;
    long long t0 = 0;
    for (int i = tid; i < n_entries && i < kAttnIdxCap; i += NT) {
      u64 v = load_agent(ent + i);
      while (!(v >> 63)) {
        if (t0 == 0) t0 = wall_clock64();
        __builtin_amdgcn_s_sleep(8);
        v = load_agent(ent + i);
        if (!(v >> 63) && wall_clock64() - t0 > a.wait_limit) { failed = 1; break; }
      }
      const int slot16 = (int)((v >> 32) & 0xffffu);
      sm.page[i] = (int32_t)(u32)v;
      sm.slot[i] = slot16 == 0xffff ? -1 : slot16;
    }
    if (failed) sm.is_last = -1;
    __syncthreads();
    if (sm.is_last < 0) return -1;
    if (inputs_ready_tick != nullptr) *inputs_ready_tick = wall_clock64();
  } else {
    if (idx_in_lds) {
      for (int i = tid; i < n_entries; i += NT) {
        sm.page[i] = sel[first + i];
        sm.slot[i] = slots[first + i];
      }
    }
    __syncthreads();
  }

  // software pipeline: three tile buffers rotate, so the operands of the next two tiles of this
  // wave (16 KiB) are in flight while one tile is computed
  struct Tile { uint4 k[4], v[4]; u32 valid; };        // valid: bit i = token i of the tile takes part
  auto issue = [&](Tile& tl, int t) {
    tl.valid = 0;
    if (t >= n_tiles) return;
    if (PACKED) {
      // lane (i, g): K units of token i of the tile = token i % P of entry i / P; V units of tokens
      // 4g..4g+3 = token group (4g % P) / 4 of entry 4g / P
      auto entry = [&](int e, int& page, int& slot) {
        page = -1; slot = -1;
        if (e < n_entries) {
          if (idx_in_lds) { page = sm.page[e]; slot = sm.slot[e]; }
          else { page = sel[first + e]; slot = slots[first + e]; }
        }
        if (slot >= a.Cmax) slot = -1;
      };
      const int e0 = t * pages_per_tile;
      int kp, ks, vp, vs;
      entry(e0 + j / a.P, kp, ks);
      entry(e0 + (4 * g) / a.P, vp, vs);
      const int ktok = j % a.P;
      const bool kok = kp >= 0 && ks >= 0 && kp * a.P + ktok < seq;
      // the tile's valid tokens: lanes 0..15 (g = 0) speak for tokens 0..15
      const u32 valid = (u32)(__ballot(kok) & 0xffffull);
      tl.valid = valid;
      if (valid == 0) return;
#pragma unroll
      for (int c = 0; c < 4; ++c) { tl.k[c] = make_uint4(0u, 0u, 0u, 0u); tl.v[c] = make_uint4(0u, 0u, 0u, 0u); }
      if (kok) {
        const char* kb = pool_u + (size_t)ks * a.page_bytes + (size_t)(g * a.P + ktok) * 16;
#pragma unroll
        for (int c = 0; c < 4; ++c) tl.k[c] = load_stream16(kb + (size_t)c * 4 * a.P * 16);
      }
      if (vp >= 0 && vs >= 0 && ((valid >> (4 * g)) & 15u)) {
        const int groups = a.P >> 2, tg = ((4 * g) % a.P) >> 2;
        const char* vb = pool_u + (size_t)vs * a.page_bytes + (size_t)a.P * kRowBytes + (size_t)(tg * 16 + j) * 16;
#pragma unroll
        for (int c = 0; c < 4; ++c) tl.v[c] = load_stream16(vb + (size_t)c * groups * 256);
      }
      return;
    }
    const int e = t / tiles_per_page, tile = t % tiles_per_page;
    int page, slot;
    if (idx_in_lds) {
      page = sm.page[e];
      slot = sm.slot[e];
    } else {
      page = sel[first + e];
      slot = slots[first + e];
    }
    page = __builtin_amdgcn_readfirstlane(page);
    slot = __builtin_amdgcn_readfirstlane(slot);
    if (page < 0 || slot < 0 || slot >= a.Cmax) return;
    int ntok = seq - page * a.P - tile * 16;
    ntok = ntok < 16 ? ntok : 16;
    if (ntok <= 0) return;
    tl.valid = ntok >= 16 ? 0xffffu : ((1u << ntok) - 1u);
    const uint4* tb = reinterpret_cast<const uint4*>(pool_u + (size_t)slot * a.page_bytes + (size_t)tile * kTileBytes) + lane;
#pragma unroll
    for (int c = 0; c < 4; ++c) tl.k[c] = load_stream16(tb + c * 64);
#pragma unroll
    for (int c = 0; c < 4; ++c) tl.v[c] = load_stream16(tb + 256 + c * 64);
  };
  auto compute = [&](Tile& tl) {
    const u32 valid = tl.valid;
    if (valid == 0) return;
    const u32 mine = (valid >> (4 * g)) & 15u;          // this lane's four tokens 4g..4g+3
    if (valid != 0xffffu) {
      // a tile with tokens that take no part (the ragged end of a sequence, whose slot holds whatever
      // the store had there since a page is copied whole; with PACKED also a missing page): a
      // probability of zero does not silence a NaN or an infinity, so those tokens' V elements are
      // blanked.  Lane (., g) holds tokens 4g..4g+3 of a dim in each half of a V fragment, two
      // tokens per 32-bit word.
      const u32 m0 = ((mine & 1u) ? 0x0000ffffu : 0u) | ((mine & 2u) ? 0xffff0000u : 0u);
      const u32 m1 = ((mine & 4u) ? 0x0000ffffu : 0u) | ((mine & 8u) ? 0xffff0000u : 0u);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        tl.v[c].x &= m0; tl.v[c].y &= m1;
        tl.v[c].z &= m0; tl.v[c].w &= m1;
      }
    }
    f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c) s = mfma_qk<BF16>(tl.k[c], LEAN ? sm.qf[c][lane] : qfrag[c], s);
    float x[4];
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[e] = ((mine >> e) & 1u) ? s[e] * a.scale_log2 : -INFINITY;
      mx = fmaxf(mx, x[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float m_new = fmaxf(m, mx);                // finite: some token of the tile is valid
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
  if (LEAN) {
    Tile ta, tb2;
    issue(ta, w);
    for (int t = w; t < n_tiles; t += 2 * NW) {
      issue(tb2, t + NW);
      compute(ta);
      issue(ta, t + 2 * NW);
      compute(tb2);
    }
  } else {
    Tile ta, tb2, tc;
    issue(ta, w);
    issue(tb2, w + NW);
    for (int t = w; t < n_tiles; t += 3 * NW) {
      issue(tc, t + 2 * NW);
      compute(ta);
      issue(ta, t + 3 * NW);
      compute(tb2);
      issue(tb2, t + 4 * NW);
      compute(tc);
    }
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
  return finish_split<GT, NT>(a, sm, u, split) ? 1 : 0;
}

}  // namespace kvd
