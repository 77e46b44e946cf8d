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
// Pages of any other size keep the natural layout of the host store: K[P][D] then V[P][D].
#pragma once

namespace kvd {
constexpr int kTileTokens = 16;
constexpr int kTileBytes = 2 * kTileTokens * 128 * 2;   // 8192
constexpr int kTilePartBytes = kTileBytes / 2;          // 4096
}  // namespace kvd
