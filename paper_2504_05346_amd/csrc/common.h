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

// Helper streams and their events are host objects that cost tens of microseconds to create
// and whose destruction waits for the stream to drain (which would stall the host inside every
// call).  They are therefore kept: a call borrows a context (one stream of default priority and
// as many events as it needs) from a per-process pool and hands it back on return; contexts are
// created on demand, one set per device and per concurrently running call, and live until the
// process ends.  A context is handed back only after its work has been joined into the
// caller's stream, so the next borrower's work is merely queued behind it.
struct StreamCtx {
  int device = -1;
  hipStream_t stream = nullptr;
  hipEvent_t* ev = nullptr;
  int nev = 0, cap = 0;
};
StreamCtx* stream_ctx_acquire(int n_events);  // nullptr on failure (api.hip)
void stream_ctx_release(StreamCtx* c);

// A helper stream (default priority) for the duration of one call, forked from and joined back
// into the caller's stream with events; it runs a long, throughput-bound update next to a chain
// of short, latency-bound kernels.
//   fork(i)    the helper waits for everything the caller's stream holds now (event i)
//   record(i)  event i <- everything the helper holds now; no launch on the helper may follow
//              a record without a new fork
//   join(i)    the caller's stream waits for event i
// If the object is destroyed while forked work has not been joined (an error return between a
// fork and its join), the destructor joins it first, so that the caller's stream never runs
// ahead of kernels that still use the caller's buffers.
// inline_mode: there is no helper: `stream` IS the caller's stream and fork / record / join do
// nothing (one in-order stream runs the kernels in the order the host enqueues them, and that
// order respects every dependency the events express).  Nothing is created or borrowed.
class AuxStream {
 public:
  hipStream_t stream = nullptr;
  bool ok = false;
  AuxStream(hipStream_t caller, int n_events, bool inline_mode)
      : caller_(caller), inline_(inline_mode || n_events <= 0) {
    if (inline_) {  // also when no fork will happen
      stream = caller;
      ok = true;
      return;
    }
    ctx_ = stream_ctx_acquire(n_events + 1);  // the last event serves the destructor
    if (!ctx_) return;
    stream = ctx_->stream;
    nev_ = n_events + 1;
    ok = true;
  }
  thanos_status fork(int i) {
    if (inline_) return THANOS_OK;
    if (i < 0 || i >= nev_ - 1) return THANOS_ERR_HIP;
    if (hipEventRecord(ctx_->ev[i], caller_) != hipSuccess) return THANOS_ERR_HIP;
    if (hipStreamWaitEvent(stream, ctx_->ev[i], 0) != hipSuccess) return THANOS_ERR_HIP;
    open_ = true;
    last_rec_ = -1;
    return THANOS_OK;
  }
  thanos_status record(int i) {
    if (inline_) return THANOS_OK;
    if (i < 0 || i >= nev_ - 1) return THANOS_ERR_HIP;
    if (hipEventRecord(ctx_->ev[i], stream) != hipSuccess) return THANOS_ERR_HIP;
    last_rec_ = i;
    return THANOS_OK;
  }
  thanos_status join(int i) {
    if (inline_) return THANOS_OK;
    if (i < 0 || i >= nev_ - 1) return THANOS_ERR_HIP;
    if (hipStreamWaitEvent(caller_, ctx_->ev[i], 0) != hipSuccess) return THANOS_ERR_HIP;
    if (i == last_rec_) open_ = false;
    return THANOS_OK;
  }
  ~AuxStream() {
    if (inline_ || !ctx_) return;
    if (open_ && hipEventRecord(ctx_->ev[nev_ - 1], stream) == hipSuccess)
      (void)hipStreamWaitEvent(caller_, ctx_->ev[nev_ - 1], 0);
    stream_ctx_release(ctx_);
  }
  AuxStream(const AuxStream&) = delete;
  AuxStream& operator=(const AuxStream&) = delete;

 private:
  hipStream_t caller_;
  StreamCtx* ctx_ = nullptr;
  int nev_ = 0;
  bool inline_;
  bool open_ = false;  // forked work that no join covers yet
  int last_rec_ = -1;  // event of the last record since the last fork
};
// Diagnostic phase timing of one call: mark(p) records a timing event on the stream and says
// "what follows belongs to phase p"; collect() waits for the stream and adds the time between
// consecutive marks to the phase of the earlier one.  A null pointer or a disabled timer costs
// nothing.  Only meaningful when all kernels of the call run on the one stream.
class PhaseTimer {
 public:
  explicit PhaseTimer(hipStream_t s) : s_(s) {}
  void mark(int phase) {
    if (n_ >= kMax - (phase < 0 ? 0 : 1)) return;  // the last slot is kept for the closing mark
    if (hipEventCreate(&ev_[n_]) != hipSuccess) return;
    (void)hipEventRecord(ev_[n_], s_);
    ph_[n_++] = phase;
  }
  thanos_status collect(float* out) {  // THANOS_N_PHASES floats
    mark(-1);
    thanos_status st = hipStreamSynchronize(s_) == hipSuccess ? THANOS_OK : THANOS_ERR_HIP;
    for (int p = 0; p < THANOS_N_PHASES; ++p) out[p] = 0.f;
    for (int i = 0; i + 1 < n_ && st == THANOS_OK; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev_[i], ev_[i + 1]) != hipSuccess) st = THANOS_ERR_HIP;
      else if (ph_[i] >= 0 && ph_[i] < THANOS_N_PHASES) out[ph_[i]] += ms;
    }
    return st;
  }
  ~PhaseTimer() {
    for (int i = 0; i < n_; ++i) (void)hipEventDestroy(ev_[i]);
  }
  PhaseTimer(const PhaseTimer&) = delete;
  PhaseTimer& operator=(const PhaseTimer&) = delete;

 private:
  static constexpr int kMax = 4096;
  hipStream_t s_;
  hipEvent_t ev_[kMax];
  int ph_[kMax];
  int n_ = 0;
};
static inline void phase_mark(PhaseTimer* t, int phase) {
  if (t) t->mark(phase);
}

#define THANOS_CHECK(expr)                 \
  do {                                     \
    thanos_status st_ = (expr);            \
    if (st_ != THANOS_OK) return st_;      \
  } while (0)
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
// single_stream: no helper streams, everything on `s` in enqueue order (nothing is created).
thanos_status factor(hipStream_t s, const float* H, int64_t b, float damping, float* U,
                     float* xnorm2, void* ws, int32_t* info, bool single_stream = false);
const float* factor_L(const void* ws, int64_t b, int64_t* ld);

// skip[i] = 1 for the n_out rows of W (c x b fp32) with the largest loss W_i H W_i^T (sweep.hip).
thanos_status row_outliers(hipStream_t s, const float* W, const float* H, int64_t c, int64_t b,
                           long long n_out, float* Hf, float* T, float* h, uint8_t* skip);

}  // namespace thanos
