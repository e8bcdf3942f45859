// Shared host/device helpers of libthanos (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/thanos.h"

#define THANOS_HIP_CHECK(expr)                      \
  do {                                              \
    hipError_t e_ = (expr);                         \
    if (e_ != hipSuccess) return THANOS_ERR_HIP;    \
  } while (0)

#define THANOS_LAUNCH_CHECK()                                   \
  do {                                                          \
    if (hipGetLastError() != hipSuccess) return THANOS_ERR_HIP; \
  } while (0)

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// A second stream (default priority) forked from and joined back into the caller's stream with
// events, used to run a long, throughput-bound update next to a chain of short, latency-bound
// kernels.  Host objects only; created and destroyed inside one call.
struct AuxStream {
  hipStream_t stream = nullptr;
  hipEvent_t* ev = nullptr;
  int nev = 0;
  bool ok = false;
  explicit AuxStream(int n_events) {
    if (hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) != hipSuccess) {
      stream = nullptr;
      return;
    }
    ev = new hipEvent_t[n_events > 0 ? n_events : 1];
    for (nev = 0; nev < n_events; ++nev)
      if (hipEventCreateWithFlags(&ev[nev], hipEventDisableTiming) != hipSuccess) return;
    ok = true;
  }
  ~AuxStream() {
    for (int i = 0; i < nev; ++i) (void)hipEventDestroy(ev[i]);
    delete[] ev;
    if (stream) (void)hipStreamDestroy(stream);
  }
  AuxStream(const AuxStream&) = delete;
  AuxStream& operator=(const AuxStream&) = delete;
};
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- internal entry points shared between translation units -------------------------------
namespace thanos {

constexpr int kFactorNB = 128;  // block size of the blocked factorisation

// C[M x N] (ldc) = beta*C + alpha * op(A) * op(B), fp32 on the matrix cores, 128x128 tiles.
//   a_kmajor: element (m,k) of op(A) is A[k*lda + m], else A[m*lda + k]
//   b_kmajor: element (k,n) of op(B) is B[k*ldb + n], else B[n*ldb + k]
//   lower_only: compute only tiles with tile_row >= tile_col (C square)
//   b_lower: op(B) (K x N, K == N) is lower triangular (zero for k < n): the reduction of an
//            output tile starts at its first column
thanos_status gemm_f32(hipStream_t s, bool a_kmajor, bool b_kmajor, int64_t M, int64_t N,
                       int64_t K, float alpha, const float* A, int64_t lda, const float* B,
                       int64_t ldb, float beta, float* C, int64_t ldc, bool lower_only,
                       bool b_lower = false);

thanos_status syrk_accumulate(hipStream_t s, float* H, int64_t b, const void* Xc,
                              thanos_dtype xdt, int64_t n_tok, int64_t ldx, float alpha);

// Damped factorisation (factor.hip).  After it the lower triangle of the reversed, padded copy
// in the workspace holds the Cholesky factor L of J H_d J (U = J L^{-1} J): factor_L() returns
// it and its leading dimension.
size_t factor_workspace_bytes(int64_t b);
thanos_status factor(hipStream_t s, const float* H, int64_t b, float damping, float* U,
                     float* xnorm2, void* ws, int32_t* info);
const float* factor_L(const void* ws, int64_t b, int64_t* ld);

// skip[i] = 1 for the n_out rows of W (c x b fp32) with the largest loss W_i H W_i^T (sweep.hip).
thanos_status row_outliers(hipStream_t s, const float* W, const float* H, int64_t c, int64_t b,
                           long long n_out, float* Hf, float* T, float* h, uint8_t* skip);

}  // namespace thanos
