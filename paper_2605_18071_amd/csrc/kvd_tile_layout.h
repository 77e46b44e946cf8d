// Slot layout for pages whose size is a multiple of 16 tokens ("tile layout").
//
// A slot holds P/16 tiles of 8 KiB; a tile covers 16 consecutive tokens of the page and consists
// of a K part and a V part of 4 KiB each, both arranged so that a wave reads them with fully
// contiguous 1 KiB loads (lane l reads 16 bytes at offset 16*l of a chunk) that are, as they
// arrive, MFMA operands:
//
//   K part, chunk c = 0..3 (1 KiB each), lane l = i + 16 g (i = token in tile, g = 0..3):
//       8 elements  K[token i][dim 32c + 8g + 0..7]
//     -> A operand of a 16x16x32 MFMA with rows = tokens, contraction over 32 dims.
//   V part, chunk c = 0..3 (1 KiB each), lane l = i + 16 g (i = dim in group, g = token group):
//       4 elements  V[token 4g + 0..3][dim 32c + i]        (first 8 bytes)
//       4 elements  V[token 4g + 0..3][dim 32c + 16 + i]   (last 8 bytes)
//     -> two A operands of 16x16x16 MFMAs with rows = dims, contraction over 16 tokens (V^T).
//
// Pages of 4 or 8 tokens ("packed layout"): 16 / P consecutive selected pages make up one 16-token
// MFMA tile, so a slot (2 * P * 256 bytes) holds its page's share of the same operands:
//
//   K part (P * 256 bytes), unit (c, g, t) at 16 * ((4c + g) * P + t):
//       8 elements  K[token t][dim 32c + 8g + 0..7]
//     -> for chunk c the P * 64 bytes of a page are contiguous, and lane (i, g) of a tile reads the
//        unit (c, g, i % P) of the tile's page i / P.
//   V part (P * 256 bytes), unit (c, tg, i) at P * 256 + 16 * ((c * P/4 + tg) * 16 + i):
//       4 elements  V[token 4tg + 0..3][dim 32c + i], then 4 elements V[token 4tg + 0..3][dim 32c + 16 + i]
//     -> lane (i, g) of a tile reads the unit (c, (4g % P) / 4, i) of the tile's page 4g / P.
//
// Pages of any other size keep the natural layout of the host store: K[P][D] then V[P][D].
#pragma once

namespace kvd {
constexpr int kTileTokens = 16;
constexpr int kTileBytes = 2 * kTileTokens * 128 * 2;   // 8192
constexpr int kTilePartBytes = kTileBytes / 2;          // 4096
// How the pages of a context are kept in their slots.
constexpr int kLayoutNatural = 0, kLayoutTiles = 1, kLayoutPacked = 2;
__host__ __device__ inline int slot_layout_of(int page_size) {
  return page_size % kTileTokens == 0 ? kLayoutTiles : ((page_size == 4 || page_size == 8) ? kLayoutPacked : kLayoutNatural);
}
}  // namespace kvd
