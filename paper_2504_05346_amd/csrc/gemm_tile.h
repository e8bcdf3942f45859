// Shared definitions of the 128x128 tile products: tile extents and the accumulator layout of
// the 32x32 MFMAs (the same for v_mfma_f32_32x32x2_f32 and v_mfma_f32_32x32x16_bf16).
//
// A workgroup owns a 128x128 tile of C; wavefronts 0..3 in a 2x2 arrangement each own
// 64x64 = 2x2 MFMA tiles (64 accumulator registers).  The product itself is in gemm_tile_x3.h.
#pragma once
#include "common.h"

namespace thanos {

constexpr int kTM = 128;
constexpr int kTN = 128;

struct TileAcc {
  f32x16 v[2][2];
};

// Row / column of accumulator element r of MFMA tile (f, g) inside the 128x128 tile.
__device__ __forceinline__ int acc_row(int wm, int f, int r, int lane) {
  return wm * 64 + f * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}
__device__ __forceinline__ int acc_col(int wn, int g, int lane) {
  return wn * 64 + g * 32 + (lane & 31);
}

__device__ __forceinline__ void acc_zero(TileAcc& acc) {
#pragma unroll
  for (int f = 0; f < 2; ++f)
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc.v[f][g][r] = 0.f;
}

}  // namespace thanos
