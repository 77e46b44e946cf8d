// Moving one 16-token tile of a page from the host store's natural layout (K[P][D] then V[P][D])
// into the tile layout of kvd_tile_layout.h, by a group of 256 threads in two phases with a
// barrier (the caller's) between them.
#pragma once
#include "kvd_device.h"
#include "kvd_tile_layout.h"

namespace kvd {

// 16-byte store into a slot.  HANDOFF: the slot is read by another workgroup of the same launch,
// so the bytes are written through with two 8-byte device-scope stores.
template <bool HANDOFF>
__device__ __forceinline__ void slot_store16(void* dst, const uint4& v) {
  if (HANDOFF) {
    u64* d = reinterpret_cast<u64*>(dst);
    store_agent(d, ((u64)v.y << 32) | v.x);
    store_agent(d + 1, ((u64)v.w << 32) | v.z);
  } else {
    *reinterpret_cast<uint4*>(dst) = v;
  }
}

// Phase A (gt = thread index in the group): fetch one 16-byte unit of K and of V (token gt / 16 of
// the tile, dims 8 (gt % 16) ..), store the K unit at its permuted place, park the V unit in LDS
// (`vt`: 16 x 128 elements, natural order).
template <bool HANDOFF = false>
__device__ __forceinline__ void tile_copy_phase_a(const char* __restrict__ src_page, int P, int tile,
                                                  char* __restrict__ dst_tile, uint16_t* vt, int gt) {
  const int row = gt >> 4, ch = gt & 15;
  const char* ksrc = src_page + ((size_t)(tile * kTileTokens + row) * kRowBytes) + ch * 16;
  const uint4 kq = *reinterpret_cast<const uint4*>(ksrc);
  const uint4 vq = *reinterpret_cast<const uint4*>(ksrc + (size_t)P * kRowBytes);
  // K: chunk c = ch / 4, lane = row + 16 * (ch % 4)
  slot_store16<HANDOFF>(dst_tile + ((ch >> 2) * 64 + (ch & 3) * 16 + row) * 16, kq);
  *reinterpret_cast<uint4*>(vt + row * kHeadDim + ch * 8) = vq;
}

// Phase B: thread gt assembles destination unit gt of the V part (chunk c, lane i + 16 g): four
// tokens 4g..4g+3 of dim 32c + i, then of dim 32c + 16 + i.
template <bool HANDOFF = false>
__device__ __forceinline__ void tile_copy_phase_b(char* __restrict__ dst_tile, const uint16_t* vt, int gt) {
  const int c = gt >> 6, g = (gt >> 4) & 3, i = gt & 15;
  uint16_t e[8];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh)
#pragma unroll
    for (int k = 0; k < 4; ++k) e[hh * 4 + k] = vt[(4 * g + k) * kHeadDim + 32 * c + 16 * hh + i];
  uint4 outv;
  outv.x = (u32)e[0] | ((u32)e[1] << 16);
  outv.y = (u32)e[2] | ((u32)e[3] << 16);
  outv.z = (u32)e[4] | ((u32)e[5] << 16);
  outv.w = (u32)e[6] | ((u32)e[7] << 16);
  slot_store16<HANDOFF>(dst_tile + kTilePartBytes + gt * 16, outv);
}

// One page of 4 or 8 tokens from the host store's natural layout into the packed layout, by the
// first 16 * P threads of a group (gt = thread index in the group), two phases with the caller's
// barrier between them.  Phase A: thread gt moves K unit gt — (c, g, t) with 4c + g = gt / P,
// t = gt % P — and parks one 16-byte unit of V in LDS (`vt`, P x 128 elements, natural order).
template <bool HANDOFF = false>
__device__ __forceinline__ void packed_copy_phase_a(const char* __restrict__ src_page, int P, char* __restrict__ dst_slot,
                                                    uint16_t* vt, int gt) {
  if (gt >= 16 * P) return;
  const int t = gt % P, cg = gt / P;
  const uint4 kq = *reinterpret_cast<const uint4*>(src_page + (size_t)t * kRowBytes + cg * 16);
  const int row = gt >> 4, ch = gt & 15;
  const uint4 vq = *reinterpret_cast<const uint4*>(src_page + (size_t)(P + row) * kRowBytes + ch * 16);
  slot_store16<HANDOFF>(dst_slot + gt * 16, kq);
  *reinterpret_cast<uint4*>(vt + row * kHeadDim + ch * 8) = vq;
}

// Phase B: thread gt assembles V unit gt = (c * P/4 + tg) * 16 + i: tokens 4tg..4tg+3 of dim
// 32c + i, then of dim 32c + 16 + i.
template <bool HANDOFF = false>
__device__ __forceinline__ void packed_copy_phase_b(int P, char* __restrict__ dst_slot, const uint16_t* vt, int gt) {
  if (gt >= 16 * P) return;
  const int i = gt & 15, q = gt >> 4, groups = P >> 2;
  const int tg = q % groups, c = q / groups;
  uint16_t e[8];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh)
#pragma unroll
    for (int k = 0; k < 4; ++k) e[hh * 4 + k] = vt[(4 * tg + k) * kHeadDim + 32 * c + 16 * hh + i];
  uint4 outv;
  outv.x = (u32)e[0] | ((u32)e[1] << 16);
  outv.y = (u32)e[2] | ((u32)e[3] << 16);
  outv.z = (u32)e[4] | ((u32)e[5] << 16);
  outv.w = (u32)e[6] | ((u32)e[7] << 16);
  slot_store16<HANDOFF>(dst_slot + (size_t)P * kRowBytes + gt * 16, outv);
}

}  // namespace kvd
