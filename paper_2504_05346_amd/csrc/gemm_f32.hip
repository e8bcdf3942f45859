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
  int vec_a, vec_b, vec_c;
  int b_lower;  // op(B) is lower triangular: the reduction starts at the tile's first column
};

template <bool AK, bool BK>
__global__ __launch_bounds__(kXThreads, 4) void k_gemm_f32(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) char sm[];
  const int tn = blockIdx.x, tm = blockIdx.y;
  if (g.lower_only && tn > tm) return;
  const int m0 = tm * kTM, n0 = tn * kTN;
  const int m_ext = min(kTM, g.M - m0), n_ext = min(kTN, g.N - n0);
  const float* A = AK ? g.A + m0 : g.A + (int64_t)m0 * g.lda;
  const float* B = BK ? g.B + n0 : g.B + (int64_t)n0 * g.ldb;
  TileAcc acc;
  acc_zero(acc);
  gemm_tile_x3<AK, BK>(acc, sm, A, g.lda, m_ext, B, g.ldb, n_ext, g.b_lower ? n0 : 0, g.K, g.vec_a,
                       g.vec_b);
  const float* T = x3_stage_tile(acc, sm);
  // row pass: wavefront w takes rows w, w + 8, ..., lane l the columns 2l, 2l + 1
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = 2 * lane;
  float* Cg = g.C + (int64_t)m0 * g.ldc + n0 + c0;
  if (m_ext == kTM && n_ext == kTN && g.vec_c) {  // whole tile, 8-byte aligned pairs
    float2 old[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
      old[i] = g.beta != 0.f ? *reinterpret_cast<const float2*>(Cg + (int64_t)(wave + 8 * i) * g.ldc)
                             : make_float2(0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float2 t = *reinterpret_cast<const float2*>(T + (wave + 8 * i) * kXCLd + c0);
      *reinterpret_cast<float2*>(Cg + (int64_t)(wave + 8 * i) * g.ldc) =
          make_float2(g.beta * old[i].x + g.alpha * t.x, g.beta * old[i].y + g.alpha * t.y);
    }
  } else {
    for (int i = 0; i < 16; ++i) {
      const int row = wave + 8 * i;
      if (row >= m_ext) break;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        if (c0 + e < n_ext) {
          float* p = Cg + (int64_t)row * g.ldc + e;
          const float o = g.beta != 0.f ? *p : 0.f;
          *p = g.beta * o + g.alpha * T[row * kXCLd + c0 + e];
        }
      }
    }
  }
}

static inline bool vec_ok(const float* p, int64_t ld) {
  return (reinterpret_cast<uintptr_t>(p) % 16 == 0) && (ld % 4 == 0);
}

thanos_status gemm_f32(hipStream_t s, bool a_kmajor, bool b_kmajor, int64_t M, int64_t N,
                       int64_t K, float alpha, const float* A, int64_t lda, const float* B,
                       int64_t ldb, float beta, float* C, int64_t ldc, bool lower_only,
                       bool b_lower) {
  if (M <= 0 || N <= 0) return THANOS_OK;
  GemmArgs g{A, B, C, lda, ldb, ldc, (int)M, (int)N, (int)K, alpha, beta, lower_only ? 1 : 0,
             vec_ok(A, lda) ? 1 : 0, vec_ok(B, ldb) ? 1 : 0,
             (reinterpret_cast<uintptr_t>(C) % 8 == 0 && ldc % 2 == 0) ? 1 : 0, b_lower ? 1 : 0};
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
