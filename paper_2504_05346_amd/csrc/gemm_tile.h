// 128x128 fp32 tile product on the CDNA4 matrix cores (v_mfma_f32_32x32x2_f32).
//
// One workgroup of 256 threads (4 wavefronts, 2x2) owns a 128x128 tile of C; each wavefront
// owns 64x64 = 2x2 MFMA tiles (64 accumulator registers).  Slabs of 16 k-values of A and B are
// staged through LDS in k-major order (a[k][m], b[k][n]) so that the MFMA operand fetch is a
// bank-conflict-free 32-bit read with consecutive lanes on consecutive m (or n).  Global loads
// of the next slab are issued before the products of the current one (register prefetch,
// two LDS buffers, one barrier per slab).
#pragma once
#include "common.h"

namespace thanos {

constexpr int kTM = 128;
constexpr int kTN = 128;
constexpr int kTK = 16;
constexpr int kLdsLd = 132;  // 128 + 4 floats: rows stay 16-byte aligned, banks are skewed

struct GemmSmem {
  float a[2][kTK][kLdsLd];
  float b[2][kTK][kLdsLd];
};

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

// One operand slab (16 k-values x 128 m-values) held in registers between global load and
// LDS store: two float4 per thread.
struct SlabRegs {
  float4 v[2];
};

// kmajor:  element (m, k) at P[k*ld + m];  else at P[m*ld + k].
// ext = number of valid m (rows beyond it read as 0); K = total k extent (k >= K reads as 0).
template <bool KMAJOR>
__device__ __forceinline__ void slab_load(SlabRegs& r, const float* __restrict__ P, int64_t ld,
                                          int ext, int k0, int K, bool vec_ok, int tid) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int idx = tid + 256 * u;
    float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
    if (KMAJOR) {
      const int k = k0 + (idx >> 5);
      const int m4 = (idx & 31) * 4;
      if (k < K && m4 < ext) {
        const float* p = P + (int64_t)k * ld + m4;
        if (vec_ok && m4 + 3 < ext) {
          val = *reinterpret_cast<const float4*>(p);
        } else {
          val.x = p[0];
          if (m4 + 1 < ext) val.y = p[1];
          if (m4 + 2 < ext) val.z = p[2];
          if (m4 + 3 < ext) val.w = p[3];
        }
      }
    } else {
      const int m = idx >> 2;
      const int k = k0 + (idx & 3) * 4;
      if (m < ext && k < K) {
        const float* p = P + (int64_t)m * ld + k;
        if (vec_ok && k + 3 < K) {
          val = *reinterpret_cast<const float4*>(p);
        } else {
          val.x = p[0];
          if (k + 1 < K) val.y = p[1];
          if (k + 2 < K) val.z = p[2];
          if (k + 3 < K) val.w = p[3];
        }
      }
    }
    r.v[u] = val;
  }
}

template <bool KMAJOR>
__device__ __forceinline__ void slab_store(float (*s)[kLdsLd], const SlabRegs& r, int tid) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int idx = tid + 256 * u;
    if (KMAJOR) {
      const int k = idx >> 5;
      const int m4 = (idx & 31) * 4;
      *reinterpret_cast<float4*>(&s[k][m4]) = r.v[u];
    } else {
      const int m = idx >> 2;
      const int k = (idx & 3) * 4;
      s[k + 0][m] = r.v[u].x;
      s[k + 1][m] = r.v[u].y;
      s[k + 2][m] = r.v[u].z;
      s[k + 3][m] = r.v[u].w;
    }
  }
}

// acc += op(A)[0:128, kbeg:kend] * op(B)[kbeg:kend, 0:128].
// A and B point at the tile origin (row 0 / column 0 of the tile, k = 0).
// kbeg must be a multiple of 4 when vec_ok is set.
template <bool A_KMAJOR, bool B_KMAJOR>
__device__ __forceinline__ void gemm_tile(TileAcc& acc, GemmSmem& sm, const float* __restrict__ A,
                                          int64_t lda, int m_ext, const float* __restrict__ B,
                                          int64_t ldb, int n_ext, int kbeg, int kend, bool vec_a,
                                          bool vec_b) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int lo = lane & 31, hi = lane >> 5;
  if (kend <= kbeg) return;
  const int nslab = (kend - kbeg + kTK - 1) / kTK;
  SlabRegs ra, rb;
  slab_load<A_KMAJOR>(ra, A, lda, m_ext, kbeg, kend, vec_a, tid);
  slab_load<B_KMAJOR>(rb, B, ldb, n_ext, kbeg, kend, vec_b, tid);
  __syncthreads();  // previous users of the LDS buffers are done
  slab_store<A_KMAJOR>(sm.a[0], ra, tid);
  slab_store<B_KMAJOR>(sm.b[0], rb, tid);
  __syncthreads();
  for (int it = 0; it < nslab; ++it) {
    const int buf = it & 1;
    if (it + 1 < nslab) {
      const int k0 = kbeg + (it + 1) * kTK;
      slab_load<A_KMAJOR>(ra, A, lda, m_ext, k0, kend, vec_a, tid);
      slab_load<B_KMAJOR>(rb, B, ldb, n_ext, k0, kend, vec_b, tid);
    }
#pragma unroll
    for (int kk = 0; kk < kTK; kk += 2) {
      const float a0 = sm.a[buf][kk + hi][wm * 64 + lo];
      const float a1 = sm.a[buf][kk + hi][wm * 64 + 32 + lo];
      const float b0 = sm.b[buf][kk + hi][wn * 64 + lo];
      const float b1 = sm.b[buf][kk + hi][wn * 64 + 32 + lo];
      acc.v[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc.v[0][0], 0, 0, 0);
      acc.v[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc.v[0][1], 0, 0, 0);
      acc.v[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc.v[1][0], 0, 0, 0);
      acc.v[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc.v[1][1], 0, 0, 0);
    }
    if (it + 1 < nslab) {
      slab_store<A_KMAJOR>(sm.a[buf ^ 1], ra, tid);
      slab_store<B_KMAJOR>(sm.b[buf ^ 1], rb, tid);
    }
    __syncthreads();
  }
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
