// Structured pruning (Alg. 2, Sec. 4.7): s = ceil(p b / (1 - alpha)) whole columns are removed
// from every non-outlier row in one shot,
//     W_R <- W_R - W_{R,Q} (Hinv[Q,Q])^{-1} Hinv[Q,:],      Hinv = (H + damping)^{-1},
// Q = the s columns of smallest loss v_j = (sum_{i in R} W_ij^2) H_jj, R = all rows but the
// ceil(alpha c) of largest loss h_i = W_i H W_i^T.
//
// How it is computed.  With sigma the ascending order of (v_j, j) and H' = H[sigma, sigma], the
// removed columns are the first s of the permuted problem, and with U' from the factorisation
// of H' (H'_d^{-1} = U'^T U'):
//     Hinv'[0:s, :]   = U'_ss^T U'[0:s, :],      Hinv'[0:s, 0:s] = U'_ss^T U'_ss,
//     Delta'          = -(W'_Q U'_ss^{-1}) U'[0:s, :],
// and U'_ss^{-1} is the index-reversed trailing s x s block of the Cholesky factor L the
// factorisation leaves in its workspace (U' = J L^{-1} J).  So: two rankings, one symmetric
// gather, the factorisation, two matrix products, one scatter.  Nothing of W is permuted in
// place; sigma only addresses columns.
#include <algorithm>
#include <cmath>

#include "common.h"

namespace thanos {

// Column losses v[j] = H[j][j] * sum over non-skipped rows of W[i][j]^2, in two steps: fp64
// partial sums over chunks of rows (blockIdx.y), then the sum of the partials in chunk order.
// The second step also clears the rank counters of k_col_rank.
__global__ __launch_bounds__(256) void k_col_loss_part(const float* __restrict__ W, int64_t c,
                                                       int64_t b, int64_t rows_per_chunk,
                                                       const uint8_t* __restrict__ skip,
                                                       double* __restrict__ part) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= b) return;
  const int64_t i0 = (int64_t)blockIdx.y * rows_per_chunk, i1 = min(c, i0 + rows_per_chunk);
  double acc = 0.0;
  for (int64_t i = i0; i < i1; ++i) {
    if (skip && skip[i]) continue;
    const double w = (double)W[i * b + j];
    acc += w * w;
  }
  part[(int64_t)blockIdx.y * b + j] = acc;
}

__global__ __launch_bounds__(256) void k_col_loss_fin(const double* __restrict__ part,
                                                      const float* __restrict__ H, int64_t b,
                                                      int nchunk, float* __restrict__ v,
                                                      int* __restrict__ rank) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= b) return;
  double acc = 0.0;
  for (int ch = 0; ch < nchunk; ++ch) acc += part[(int64_t)ch * b + j];
  v[j] = (float)(acc * (double)H[j * b + j]);
  rank[j] = 0;
}

// rank[j] = number of columns before j in ascending (v, j) order; every workgroup counts one
// chunk of 2048 competitors (blockIdx.y) for its 256 columns (integer atomics: order-free).
__global__ __launch_bounds__(256) void k_col_rank(const float* __restrict__ v, int64_t b,
                                                  int* __restrict__ rank) {
  __shared__ float vs[2048];
  const int64_t k0 = (int64_t)blockIdx.y * 2048;
  const int nk = (int)min((int64_t)2048, b - k0);
  for (int e = threadIdx.x; e < nk; e += 256) vs[e] = v[k0 + e];
  __syncthreads();
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= b) return;
  const float mine = v[j];
  int cnt = 0;
  for (int e = 0; e < nk; ++e) {
    const float o = vs[e];
    cnt += (o < mine || (o == mine && k0 + e < j)) ? 1 : 0;
  }
  if (cnt) atomicAdd(&rank[j], cnt);
}

// sigma[rank[j]] = j (rank is sigma's inverse).
__global__ __launch_bounds__(256) void k_col_order(const int* __restrict__ rank, int64_t b,
                                                   int* __restrict__ sigma) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j < b) sigma[rank[j]] = (int)j;
}

// Hp[x][y] = H_sym[sigma[x]][sigma[y]] for y <= x (H given by its lower triangle).
__global__ __launch_bounds__(256) void k_permute_sym(const float* __restrict__ H, int64_t b,
                                                     const int* __restrict__ sigma,
                                                     float* __restrict__ Hp) {
  const int64_t y = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t x = blockIdx.y;
  if (y > x || y >= b) return;
  const int64_t sx = sigma[x], sy = sigma[y];
  Hp[x * b + y] = (sx >= sy) ? H[sx * b + sy] : H[sy * b + sx];
}

// WQ[i][x] = W[i][sigma[x]], x < s.
__global__ __launch_bounds__(256) void k_gather_cols(const float* __restrict__ W, int64_t b,
                                                     const int* __restrict__ sigma, int64_t s,
                                                     float* __restrict__ WQ) {
  const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t i = blockIdx.y;
  if (x >= s) return;
  WQ[i * s + x] = W[i * b + sigma[x]];
}

// M[x][y] = L[b-1-x][b-1-y] for x <= y, else 0 (s x s): the inverse of U'_ss.
__global__ __launch_bounds__(256) void k_rev_L(const float* __restrict__ L, int64_t ld, int64_t b,
                                               int64_t s, float* __restrict__ M) {
  const int64_t y = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t x = blockIdx.y;
  if (y >= s) return;
  M[x * s + y] = (x <= y) ? L[(b - 1 - x) * ld + (b - 1 - y)] : 0.f;
}

// Non-skipped rows: column j sits at position pos = rank[j] of the permuted order;
// W[i][j] = 0 for pos < s, else -= T[i][pos]; mask accordingly.  (Threads run over the natural
// columns: W and the mask are written in whole rows, only T is gathered.)
__global__ __launch_bounds__(256) void k_struct_apply(float* __restrict__ W,
                                                      const float* __restrict__ T, int64_t b,
                                                      const int* __restrict__ rank, int64_t s,
                                                      const uint8_t* __restrict__ skip,
                                                      uint8_t* __restrict__ mask) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t i = blockIdx.y;
  if (j >= b) return;
  const int64_t idx = i * b + j;
  if (skip && skip[i]) {
    mask[idx] = 0;
    return;
  }
  const int64_t pos = rank[j];
  if (pos < s) {
    W[idx] = 0.f;
    mask[idx] = 1;
  } else {
    if (s > 0) W[idx] -= T[i * b + pos];
    mask[idx] = 0;
  }
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(__half x) { return __half2float(x); }
__device__ __forceinline__ float to_f32(__hip_bfloat16 x) { return __bfloat162float(x); }
__device__ __forceinline__ void from_f32(float x, float& o) { o = x; }
__device__ __forceinline__ void from_f32(float x, __half& o) { o = __float2half(x); }
__device__ __forceinline__ void from_f32(float x, __hip_bfloat16& o) { o = __float2bfloat16(x); }

template <typename T>
__global__ __launch_bounds__(256) void k_conv_in(const T* __restrict__ in, float* __restrict__ out,
                                                 int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = to_f32(in[i]);
}
template <typename T>
__global__ __launch_bounds__(256) void k_conv_out(const float* __restrict__ in, T* __restrict__ out,
                                                  int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) from_f32(in[i], out[i]);
}

static char* carve(char*& p, size_t bytes) {
  char* q = p;
  p += align_up(bytes, 256);
  return q;
}

size_t structured_workspace_bytes(int64_t c, int64_t b) {
  size_t n = 0;
  n += align_up((size_t)b * b * 4, 256);      // HB: symmetric H, then H', then U'_ss^{-1}
  n += align_up((size_t)c * b * 4, 256);      // T: W H, then the update in permuted order
  n += align_up((size_t)c * b * 4, 256);      // WQ
  n += align_up((size_t)c * b * 4, 256);      // Z
  n += align_up((size_t)b * b * 4, 256);      // U'
  n += 2 * align_up((size_t)b * 4, 256);      // v, xnorm2'
  n += 2 * align_up((size_t)b * 4, 256);      // sigma and its inverse
  n += align_up((size_t)c * 4, 256);          // h
  n += align_up((size_t)c, 256);              // row_skip
  n += align_up(factor_workspace_bytes(b), 256);
  return n;
}

thanos_status structured(hipStream_t st, const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                         const float* H, float damping, long long s_cols, long long n_out,
                         float* W, void* W_cast, uint8_t* mask, void* ws, int32_t* info,
                         bool single_stream) {
  char* p = reinterpret_cast<char*>(ws);
  float* HB = reinterpret_cast<float*>(carve(p, (size_t)b * b * 4));
  float* T = reinterpret_cast<float*>(carve(p, (size_t)c * b * 4));
  float* WQ = reinterpret_cast<float*>(carve(p, (size_t)c * b * 4));
  float* Z = reinterpret_cast<float*>(carve(p, (size_t)c * b * 4));
  float* U = reinterpret_cast<float*>(carve(p, (size_t)b * b * 4));
  float* v = reinterpret_cast<float*>(carve(p, (size_t)b * 4));
  float* xn2 = reinterpret_cast<float*>(carve(p, (size_t)b * 4));
  int* sigma = reinterpret_cast<int*>(carve(p, (size_t)b * 4));
  int* rank = reinterpret_cast<int*>(carve(p, (size_t)b * 4));
  float* h = reinterpret_cast<float*>(carve(p, (size_t)c * 4));
  uint8_t* skip = reinterpret_cast<uint8_t*>(carve(p, (size_t)c));
  void* fws = p;

  const int64_t n = c * b;
  const unsigned nblk = (unsigned)ceil_div(n, 256);
  if (wdt == THANOS_F32)
    hipLaunchKernelGGL(k_conv_in<float>, dim3(nblk), dim3(256), 0, st, (const float*)W_in, W, n);
  else if (wdt == THANOS_F16)
    hipLaunchKernelGGL(k_conv_in<__half>, dim3(nblk), dim3(256), 0, st, (const __half*)W_in, W, n);
  else
    hipLaunchKernelGGL(k_conv_in<__hip_bfloat16>, dim3(nblk), dim3(256), 0, st,
                       (const __hip_bfloat16*)W_in, W, n);
  THANOS_LAUNCH_CHECK();

  const uint8_t* skip_c = nullptr;
  if (n_out > 0) {
    thanos_status e = row_outliers(st, W, H, c, b, n_out, HB, T, h, skip);
    if (e != THANOS_OK) return e;
    skip_c = skip;
  }
  const unsigned bb = (unsigned)ceil_div(b, 256);
  {
    // partial sums live in the (still unused) buffer of U': nchunk * b doubles <= b * b floats
    int nchunk = (int)std::max<int64_t>(1, std::min<int64_t>(32, c / 64));
    nchunk = (int)std::min<int64_t>(nchunk, std::max<int64_t>(1, b / 2));
    const int64_t rpc = ceil_div(c, nchunk);
    double* part = reinterpret_cast<double*>(U);
    hipLaunchKernelGGL(k_col_loss_part, dim3(bb, (unsigned)nchunk), dim3(256), 0, st, W, c, b, rpc,
                       skip_c, part);
    hipLaunchKernelGGL(k_col_loss_fin, dim3(bb), dim3(256), 0, st, part, H, b, nchunk, v, rank);
    hipLaunchKernelGGL(k_col_rank, dim3(bb, (unsigned)ceil_div(b, 2048)), dim3(256), 0, st, v, b,
                       rank);
    hipLaunchKernelGGL(k_col_order, dim3(bb), dim3(256), 0, st, rank, b, sigma);
    THANOS_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(k_permute_sym, dim3(bb, (unsigned)b), dim3(256), 0, st, H, b, sigma, HB);
  THANOS_LAUNCH_CHECK();
  thanos_status e = factor(st, HB, b, damping, U, xn2, fws, info, single_stream);
  if (e != THANOS_OK) return e;
  if (s_cols > 0) {
    const int64_t s = s_cols;
    int64_t ldL = 0;
    const float* L = factor_L(fws, b, &ldL);
    hipLaunchKernelGGL(k_rev_L, dim3((unsigned)ceil_div(s, 256), (unsigned)s), dim3(256), 0, st, L,
                       ldL, b, s, HB);
    THANOS_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_gather_cols, dim3((unsigned)ceil_div(s, 256), (unsigned)c), dim3(256), 0,
                       st, W, b, sigma, s, WQ);
    THANOS_LAUNCH_CHECK();
    // Z = W_Q U'_ss^{-1}  (c x s),  T = Z U'[0:s, :]  (c x b)
    e = gemm_f32(st, false, true, c, s, s, 1.f, WQ, s, HB, s, 0.f, Z, s, false);
    if (e != THANOS_OK) return e;
    e = gemm_f32(st, false, true, c, b, s, 1.f, Z, s, U, b, 0.f, T, b, false);
    if (e != THANOS_OK) return e;
  }
  hipLaunchKernelGGL(k_struct_apply, dim3(bb, (unsigned)c), dim3(256), 0, st, W, T, b, rank,
                     (int64_t)s_cols, skip_c, mask);
  THANOS_LAUNCH_CHECK();
  if (W_cast) {
    if (wdt == THANOS_F32)
      hipLaunchKernelGGL(k_conv_out<float>, dim3(nblk), dim3(256), 0, st, W, (float*)W_cast, n);
    else if (wdt == THANOS_F16)
      hipLaunchKernelGGL(k_conv_out<__half>, dim3(nblk), dim3(256), 0, st, W, (__half*)W_cast, n);
    else
      hipLaunchKernelGGL(k_conv_out<__hip_bfloat16>, dim3(nblk), dim3(256), 0, st, W,
                         (__hip_bfloat16*)W_cast, n);
    THANOS_LAUNCH_CHECK();
  }
  return THANOS_OK;
}

}  // namespace thanos
