// fp32 matrix product (split-bf16 arithmetic on the matrix cores, see gemm_tile_x3.h), used by
// the factorisation, the sweep and the fp32 Hessian accumulation.
#include "gemm_tile_x3.h"

namespace thanos {

struct GemmArgs {
  const float* A;
  const float* B;
  float* C;
  int64_t lda, ldb, ldc;
  int M, N, K;
  float alpha, beta;
  int lower_only;
  int vec_a, vec_b;
};

template <bool AK, bool BK>
__global__ __launch_bounds__(kXThreads) void k_gemm_f32(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char sm[];
  const int tn = blockIdx.x, tm = blockIdx.y;
  if (g.lower_only && tn > tm) return;
  const int m0 = tm * kTM, n0 = tn * kTN;
  const int m_ext = min(kTM, g.M - m0), n_ext = min(kTN, g.N - n0);
  const float* A = AK ? g.A + m0 : g.A + (int64_t)m0 * g.lda;
  const float* B = BK ? g.B + n0 : g.B + (int64_t)n0 * g.ldb;
  TileAcc acc;
  acc_zero(acc);
  gemm_tile_x3<AK, BK>(acc, sm, A, g.lda, m_ext, B, g.ldb, n_ext, 0, g.K, g.vec_a, g.vec_b);
  if (threadIdx.x >= 256) return;  // producer wavefronts hold no result
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // Per 32x32 MFMA tile: 16 loads, then 16 stores.  A load placed right behind a store to the
  // same array would have to wait for it, which serialises 64 memory round trips per thread.
#pragma unroll
  for (int f = 0; f < 2; ++f)
#pragma unroll
    for (int gg = 0; gg < 2; ++gg) {
      const int col = acc_col(wn, gg, lane);
      float old[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = acc_row(wm, f, r, lane);
        old[r] = (g.beta != 0.f && row < m_ext && col < n_ext)
                     ? g.C[(int64_t)(m0 + row) * g.ldc + (n0 + col)]
                     : 0.f;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = acc_row(wm, f, r, lane);
        if (row < m_ext && col < n_ext)
          g.C[(int64_t)(m0 + row) * g.ldc + (n0 + col)] =
              g.beta * old[r] + g.alpha * acc.v[f][gg][r];
      }
    }
}

static inline bool vec_ok(const float* p, int64_t ld) {
  return (reinterpret_cast<uintptr_t>(p) % 16 == 0) && (ld % 4 == 0);
}

thanos_status gemm_f32(hipStream_t s, bool a_kmajor, bool b_kmajor, int64_t M, int64_t N,
                       int64_t K, float alpha, const float* A, int64_t lda, const float* B,
                       int64_t ldb, float beta, float* C, int64_t ldc, bool lower_only) {
  if (M <= 0 || N <= 0) return THANOS_OK;
  GemmArgs g{A, B, C, lda, ldb, ldc, (int)M, (int)N, (int)K, alpha, beta, lower_only ? 1 : 0,
             vec_ok(A, lda) ? 1 : 0, vec_ok(B, ldb) ? 1 : 0};
  dim3 grid((unsigned)ceil_div(N, kTN), (unsigned)ceil_div(M, kTM));
  void (*kern)(GemmArgs);
  if (!a_kmajor && !b_kmajor) kern = k_gemm_f32<false, false>;
  else if (!a_kmajor && b_kmajor) kern = k_gemm_f32<false, true>;
  else if (a_kmajor && b_kmajor) kern = k_gemm_f32<true, true>;
  else kern = k_gemm_f32<true, false>;
  THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kXSmemBytes));
  hipLaunchKernelGGL(kern, grid, dim3(kXThreads), kXSmemBytes, s, g);
  THANOS_LAUNCH_CHECK();
  return THANOS_OK;
}

}  // namespace thanos
