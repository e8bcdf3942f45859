// C ABI of libthanos: argument checks and orchestration only; all arithmetic is in the kernels.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <vector>

#include "common.h"

namespace thanos {
size_t sweep_workspace_bytes(int64_t c, int64_t b, int B, bool outliers, int smax, bool comp);
bool sweep_uses_complement(const thanos_prune_opts* o, int64_t b);
thanos_status sweep(hipStream_t s, const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                    const float* H, const float* U, const float* xnorm2,
                    const thanos_prune_opts* o, long long r_total, long long n_out, float* W,
                    void* W_cast, uint8_t* mask, void* ws, int32_t* info, bool single_stream,
                    PhaseTimer* pt, const float* Lfac, int64_t ldL, bool prepared);
thanos_status sweep_prepare(hipStream_t s, const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                            const float* H, const thanos_prune_opts* o, long long n_out, float* W,
                            void* ws);
size_t structured_workspace_bytes(int64_t c, int64_t b);
thanos_status structured(hipStream_t st, const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                         const float* H, float damping, long long s_cols, long long n_out,
                         float* W, void* W_cast, uint8_t* mask, void* ws, int32_t* info,
                         bool single_stream);
__global__ void k_zero_info(int32_t* info) { *info = 0; }
}  // namespace thanos

using namespace thanos;

// ---- pool of helper-stream contexts (see common.h) ----------------------------------------
namespace {
struct StreamPool {
  std::mutex mu;
  std::vector<StreamCtx*> idle;
};
StreamPool& stream_pool() {
  static StreamPool* p = new StreamPool;  // never destroyed: no HIP call at process exit
  return *p;
}
}  // namespace

StreamCtx* stream_ctx_acquire(int n_events) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return nullptr;
  StreamCtx* c = nullptr;
  {
    StreamPool& pool = stream_pool();
    std::lock_guard<std::mutex> guard(pool.mu);
    for (size_t i = 0; i < pool.idle.size(); ++i)
      if (pool.idle[i]->device == dev) {
        c = pool.idle[i];
        pool.idle.erase(pool.idle.begin() + (long)i);
        break;
      }
  }
  if (!c) {
    c = new StreamCtx;
    c->device = dev;
    if (hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking) != hipSuccess) {
      delete c;
      return nullptr;
    }
  }
  if (c->cap < n_events) {
    hipEvent_t* ev = new hipEvent_t[n_events];
    for (int i = 0; i < c->nev; ++i) ev[i] = c->ev[i];
    delete[] c->ev;
    c->ev = ev;
    c->cap = n_events;
  }
  while (c->nev < n_events) {
    if (hipEventCreateWithFlags(&c->ev[c->nev], hipEventDisableTiming) != hipSuccess) {
      stream_ctx_release(c);  // keeps what exists
      return nullptr;
    }
    ++c->nev;
  }
  return c;
}

void stream_ctx_release(StreamCtx* c) {
  if (!c) return;
  StreamPool& pool = stream_pool();
  std::lock_guard<std::mutex> guard(pool.mu);
  pool.idle.push_back(c);
}

// Workspace of thanos_prune_layer_noalloc: one array per GPU, held from the moment the library's
// code is loaded on that GPU until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address it stands for differs from GPU to GPU.
static __device__ __align__(256) unsigned char scratch[THANOS_NOALLOC_SCRATCH_BYTES];

// Device address of `scratch` on the current device, looked up once per device.
static thanos_status scratch_of_current_device(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return THANOS_ERR_HIP;
  std::lock_guard<std::mutex> guard(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return THANOS_ERR_HIP;
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return THANOS_OK;
}

static bool dtype_ok(int d) { return d == THANOS_F32 || d == THANOS_F16 || d == THANOS_BF16; }

// ---- counts derived from p and alpha ------------------------------------------------------
// p and alpha are read as the decimal they print as: the shortest decimal string that converts
// back to the same double (0.6 means 6/10, not the binary value just below it), and the counts
// floor(p*c*b), ceil(alpha*c), ceil(p*b/(1-alpha)) are then evaluated in exact integer
// arithmetic.
typedef unsigned __int128 u128;

struct Decimal {  // value = mant / 10^scale
  unsigned long long mant;
  int scale;
};

static Decimal shortest_decimal(double x) {
  char buf[48];
  for (int digits = 1; digits <= 17; ++digits) {
    snprintf(buf, sizeof buf, "%.*e", digits - 1, x);  // d.ddde[+-]xx, correctly rounded
    if (strtod(buf, nullptr) == x) break;
  }
  Decimal d{0ull, 0};
  const char* q = buf;
  bool frac = false;
  for (; *q && *q != 'e'; ++q) {
    if (*q == '.') {
      frac = true;
      continue;
    }
    if (*q < '0' || *q > '9') continue;  // sign (callers pass x >= 0)
    d.mant = d.mant * 10ull + (unsigned long long)(*q - '0');
    if (frac) ++d.scale;
  }
  if (*q == 'e') d.scale -= atoi(q + 1);
  while (d.scale < 0) {  // x < 1 in every caller, so this only normalises "0e+00"
    d.mant *= 10ull;
    ++d.scale;
  }
  while (d.scale > 0 && d.mant % 10ull == 0ull) {
    d.mant /= 10ull;
    --d.scale;
  }
  return d;
}

static bool pow10_u128(int e, u128* out) {
  if (e < 0 || e > 38) return false;
  u128 v = 1;
  for (int i = 0; i < e; ++i) v *= 10;
  *out = v;
  return true;
}

// r = floor(p*c*b)  (Alg. 1 "r <- pcb", problem statement: floor)
static long long num_to_remove(double p, int64_t c, int64_t b) {
  const Decimal d = shortest_decimal(p);
  u128 den;
  if (!pow10_u128(d.scale, &den)) return 0;  // p < 1e-38
  return (long long)((u128)d.mant * (u128)c * (u128)b / den);  // < 2^57 * 2^24 * 2^16
}

// Number of outlier rows, ceil(alpha*c)  (Sec. 4.7 "Outlier rows")
static long long num_outlier_rows(double alpha, int64_t c) {
  if (!(alpha > 0.0)) return 0;
  const Decimal d = shortest_decimal(alpha);
  u128 den;
  if (!pow10_u128(d.scale, &den)) return 1;  // 0 < alpha*c < 1
  const long long n = (long long)(((u128)d.mant * (u128)c + den - 1) / den);
  return n > c ? c : n;
}

static u128 gcd_u128(u128 a, u128 b) {
  while (b != 0) {
    const u128 t = a % b;
    a = b;
    b = t;
  }
  return a;
}

// Columns removed by the structured algorithm, ceil(p*b/(1-alpha))  (Alg. 2).
static long long num_columns_to_remove(double p, double alpha, int64_t b) {
  const Decimal dp = shortest_decimal(p), da = shortest_decimal(alpha > 0.0 ? alpha : 0.0);
  u128 tp, ta;
  if (dp.mant == 0) return 0;
  if (pow10_u128(dp.scale, &tp) && pow10_u128(da.scale, &ta) && (u128)da.mant < ta) {
    // p*b/(1-alpha) = (P*b*Ta) / (Tp*(Ta-A)); reduce before multiplying
    u128 n1 = (u128)dp.mant * (u128)b, d1 = tp, n2 = ta, d2 = ta - (u128)da.mant;
    u128 g = gcd_u128(n1, d1);
    n1 /= g, d1 /= g;
    g = gcd_u128(n2, d2);
    n2 /= g, d2 /= g;
    g = gcd_u128(n1, d2);
    n1 /= g, d2 /= g;
    g = gcd_u128(n2, d1);
    n2 /= g, d1 /= g;
    u128 num, den;
    if (!__builtin_mul_overflow(n1, n2, &num) && !__builtin_mul_overflow(d1, d2, &den)) {
      const u128 q = (num + den - 1) / den;
      return q > (u128)1 << 62 ? (long long)1 << 62 : (long long)q;
    }
  }
  // decimals too long for 128 bits: plain extended-precision evaluation
  const long double x = (long double)p * (long double)b / (1.0L - (long double)alpha);
  const long long n = (long long)ceill(x);
  return n < 0 ? 0 : n;
}

// Largest number of weights a row can lose in one block (= unknowns of its system).
static int max_unknowns(const thanos_prune_opts* o) {
  return (o->mode == THANOS_NM && !o->mask_in) ? o->block_size / o->m * o->n : o->block_size;
}

static thanos_status check_opts(const thanos_prune_opts* o, int64_t c, int64_t b) {
  if (!o) return THANOS_ERR_INVALID_ARG;
  if (o->mode != THANOS_UNSTRUCTURED && o->mode != THANOS_NM && o->mode != THANOS_STRUCTURED)
    return THANOS_ERR_INVALID_ARG;
  if (!(o->damping >= 0.f)) return THANOS_ERR_INVALID_ARG;
  if (!(o->outlier_fraction >= 0.0 && o->outlier_fraction < 1.0)) return THANOS_ERR_INVALID_ARG;
  if (o->mode == THANOS_STRUCTURED) {
    if (!(o->sparsity >= 0.0 && o->sparsity < 1.0)) return THANOS_ERR_INVALID_ARG;
    if (num_columns_to_remove(o->sparsity, o->outlier_fraction, b) > b)
      return THANOS_ERR_INVALID_ARG;  // p / (1 - alpha) > 1
    if (o->factor_in || o->mask_in) return THANOS_ERR_UNSUPPORTED;  // the factor is of H[sigma,sigma]
    if (c > 65535) return THANOS_ERR_UNSUPPORTED;  // its row-wise kernels put the row in grid.y
    return THANOS_OK;
  }
  if (o->block_size < 1) return THANOS_ERR_INVALID_ARG;
  if (o->mode == THANOS_UNSTRUCTURED) {
    if (!(o->sparsity >= 0.0 && o->sparsity < 1.0)) return THANOS_ERR_INVALID_ARG;
  } else {
    if (o->n <= 0 || o->m <= o->n) return THANOS_ERR_INVALID_ARG;
    if (o->block_size % o->m != 0 || b % o->m != 0) return THANOS_ERR_INVALID_ARG;
    if (o->m > 16) return THANOS_ERR_UNSUPPORTED;
  }
  if (o->factor_in && !o->xnorm2_in) return THANOS_ERR_INVALID_ARG;
  if (o->outlier_fraction > 0.0 && o->mode != THANOS_NM) return THANOS_ERR_UNSUPPORTED;
  // a given mask already says which rows are pruned; the outlier rows are a selection rule
  if (o->outlier_fraction > 0.0 && o->mask_in) return THANOS_ERR_UNSUPPORTED;
  // the per-row systems must fit the solver: at most 2048 unknowns, blocks of at most 4096 columns
  if (o->block_size > 4096 || max_unknowns(o) > 2048) return THANOS_ERR_UNSUPPORTED;
  (void)c;
  return THANOS_OK;
}

extern "C" {

const char* thanos_status_string(thanos_status s) {
  switch (s) {
    case THANOS_OK: return "ok";
    case THANOS_ERR_INVALID_ARG: return "invalid argument";
    case THANOS_ERR_UNSUPPORTED: return "unsupported configuration";
    case THANOS_ERR_WORKSPACE: return "workspace too small";
    case THANOS_ERR_NOT_SPD: return "matrix not positive definite";
    case THANOS_ERR_HIP: return "HIP runtime error";
    case THANOS_ERR_TOO_LARGE: return "problem exceeds the static scratch of the no-allocation entry point";
  }
  return "unknown status";
}

thanos_status thanos_hessian_accumulate(float* H, int64_t b, const void* Xc, thanos_dtype xdt,
                                        int64_t n_tok, int64_t ldx, float alpha, void* stream) {
  if (!H || b <= 0 || n_tok < 0 || !dtype_ok(xdt)) return THANOS_ERR_INVALID_ARG;
  if (n_tok == 0) return THANOS_OK;
  if (!Xc || ldx < b) return THANOS_ERR_INVALID_ARG;
  if (b > (int64_t)1 << 20) return THANOS_ERR_UNSUPPORTED;
  return syrk_accumulate(reinterpret_cast<hipStream_t>(stream), H, b, Xc, xdt, n_tok, ldx, alpha);
}

size_t thanos_factor_workspace_bytes(int64_t b) {
  if (b <= 0) return 0;
  return factor_workspace_bytes(b);
}

thanos_status thanos_factor(const float* H, int64_t b, float damping, float* U, float* xnorm2,
                            void* ws, size_t ws_bytes, int32_t* info_dev, void* stream) {
  if (!H || !U || !xnorm2 || !info_dev || b <= 0 || !(damping >= 0.f)) return THANOS_ERR_INVALID_ARG;
  if (U == H) return THANOS_ERR_INVALID_ARG;
  if (b > 65535) return THANOS_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < factor_workspace_bytes(b)) return THANOS_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return THANOS_ERR_INVALID_ARG;
  return factor(reinterpret_cast<hipStream_t>(stream), H, b, damping, U, xnorm2, ws, info_dev);
}

size_t thanos_prune_workspace_bytes(int64_t c, int64_t b, const thanos_prune_opts* opts) {
  if (c <= 0 || b <= 0 || check_opts(opts, c, b) != THANOS_OK) return 0;
  if (opts->mode == THANOS_STRUCTURED) return structured_workspace_bytes(c, b);
  size_t n = sweep_workspace_bytes(c, b, opts->block_size, opts->outlier_fraction > 0.0,
                                   max_unknowns(opts), sweep_uses_complement(opts, b));
  if (!opts->factor_in) {
    n += align_up((size_t)b * b * sizeof(float), 256);  // U
    n += align_up((size_t)b * sizeof(float), 256);      // xnorm2
    n += align_up(factor_workspace_bytes(b), 256);
  }
  return n;
}

// Argument checks shared by the two sweep entry points (everything but the workspace).
static thanos_status check_prune_args(const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                                      const float* H, const thanos_prune_opts* opts,
                                      const float* W_out, const uint8_t* mask_out,
                                      const int32_t* info_dev) {
  if (!W_in || !W_out || !mask_out || !info_dev || c <= 0 || b <= 0 || !dtype_ok(wdt))
    return THANOS_ERR_INVALID_ARG;
  thanos_status st = check_opts(opts, c, b);
  if (st != THANOS_OK) return st;
  if (!opts->factor_in && !H) return THANOS_ERR_INVALID_ARG;
  if (opts->outlier_fraction > 0.0 && !H) return THANOS_ERR_INVALID_ARG;  // row losses need H
  if (opts->mode == THANOS_STRUCTURED && !H) return THANOS_ERR_INVALID_ARG;
  if (b > 65535 || c > ((int64_t)1 << 24)) return THANOS_ERR_UNSUPPORTED;
  return THANOS_OK;
}

// Factor (unless given) and sweep with `ws` as the workspace (checked by the caller).
static thanos_status prune_with_workspace(const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                                          const float* H, const thanos_prune_opts* opts,
                                          float* W_out, void* W_out_cast, uint8_t* mask_out,
                                          void* ws, int32_t* info_dev, hipStream_t s,
                                          bool single_stream) {
  if (opts->mode == THANOS_STRUCTURED) {
    if (opts->phase_ms_out) return THANOS_ERR_UNSUPPORTED;
    return structured(s, W_in, wdt, c, b, H, opts->damping,
                      num_columns_to_remove(opts->sparsity, opts->outlier_fraction, b),
                      num_outlier_rows(opts->outlier_fraction, c), W_out, W_out_cast, mask_out, ws,
                      info_dev, single_stream);
  }
  // diagnostic mode: phases timed with events, kernels serialised on the one stream
  PhaseTimer* pt = nullptr;
  struct TimerOwner {
    PhaseTimer* t = nullptr;
    ~TimerOwner() { delete t; }
  } owner;
  if (opts->phase_ms_out) {
    owner.t = pt = new PhaseTimer(s);
    single_stream = true;
  }
  phase_mark(pt, THANOS_PHASE_FACTOR);
  char* p = reinterpret_cast<char*>(ws);
  void* sweep_ws = p;
  p += sweep_workspace_bytes(c, b, opts->block_size, opts->outlier_fraction > 0.0,
                             max_unknowns(opts), sweep_uses_complement(opts, b));
  const float* U = opts->factor_in;
  const float* xn2 = opts->xnorm2_in;
  const float* Lfac = nullptr;  // lower factor of the index-reversed damped Hessian (this call's)
  int64_t ldL = 0;
  const long long r_total =
      (opts->mode == THANOS_UNSTRUCTURED) ? num_to_remove(opts->sparsity, c, b) : 0;
  const long long n_out = num_outlier_rows(opts->outlier_fraction, c);
  bool prepared = false;
  // The working copy of the weights and the ranking of the row losses need nothing from the
  // factorisation: with a factor to compute they run beside it on a helper stream (the chain
  // of diagonal blocks leaves most of the chip idle) and are joined before the sweep.
  AuxStream prep(s, (!U && !single_stream) ? 2 : 0, single_stream);
  if (!prep.ok) return THANOS_ERR_HIP;
  if (!U) {
    float* Uw = reinterpret_cast<float*>(p);
    p += align_up((size_t)b * b * sizeof(float), 256);
    float* xw = reinterpret_cast<float*>(p);
    p += align_up((size_t)b * sizeof(float), 256);
    if (!single_stream) {
      THANOS_CHECK(prep.fork(0));
      thanos_status sp = sweep_prepare(prep.stream, W_in, wdt, c, b, H, opts, n_out, W_out, sweep_ws);
      if (sp != THANOS_OK) return sp;
      THANOS_CHECK(prep.record(1));
      prepared = true;
    }
    thanos_status st = factor(s, H, b, opts->damping, Uw, xw, p, info_dev, single_stream);
    if (st != THANOS_OK) return st;
    if (prepared) THANOS_CHECK(prep.join(1));
    U = Uw;
    xn2 = xw;
    Lfac = factor_L(p, b, &ldL);
  } else {
    hipLaunchKernelGGL(k_zero_info, dim3(1), dim3(1), 0, s, info_dev);
    THANOS_LAUNCH_CHECK();
  }
  phase_mark(pt, THANOS_PHASE_PREP);
  thanos_status st = sweep(s, W_in, wdt, c, b, H, U, xn2, opts, r_total, n_out, W_out, W_out_cast,
                           mask_out, sweep_ws, info_dev, single_stream, pt, Lfac, ldL, prepared);
  if (pt) {
    const thanos_status tc = pt->collect(opts->phase_ms_out);
    if (st == THANOS_OK) st = tc;
  }
  return st;
}

thanos_status thanos_prune_layer(const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                                 const float* H, const thanos_prune_opts* opts, float* W_out,
                                 void* W_out_cast, uint8_t* mask_out, void* ws, size_t ws_bytes,
                                 int32_t* info_dev, void* stream) {
  thanos_status st = check_prune_args(W_in, wdt, c, b, H, opts, W_out, mask_out, info_dev);
  if (st != THANOS_OK) return st;
  if (!ws || ws_bytes < thanos_prune_workspace_bytes(c, b, opts)) return THANOS_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return THANOS_ERR_INVALID_ARG;
  return prune_with_workspace(W_in, wdt, c, b, H, opts, W_out, W_out_cast, mask_out, ws, info_dev,
                              reinterpret_cast<hipStream_t>(stream), false);
}

thanos_status thanos_prune_layer_noalloc(const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                                         const float* H, const thanos_prune_opts* opts,
                                         float* W_out, void* W_out_cast, uint8_t* mask_out,
                                         int32_t* info_dev, void* stream) {
  thanos_status st = check_prune_args(W_in, wdt, c, b, H, opts, W_out, mask_out, info_dev);
  if (st != THANOS_OK) return st;
  if (opts->phase_ms_out) return THANOS_ERR_UNSUPPORTED;  // the diagnostic mode creates events
  if (thanos_prune_workspace_bytes(c, b, opts) > (size_t)THANOS_NOALLOC_SCRATCH_BYTES)
    return THANOS_ERR_TOO_LARGE;
  void* ws = nullptr;
  st = scratch_of_current_device(&ws);
  if (st != THANOS_OK) return st;
  // single stream: no helper streams or events are created; the kernels run in enqueue order
  return prune_with_workspace(W_in, wdt, c, b, H, opts, W_out, W_out_cast, mask_out, ws, info_dev,
                              reinterpret_cast<hipStream_t>(stream), true);
}

}  // extern "C"
