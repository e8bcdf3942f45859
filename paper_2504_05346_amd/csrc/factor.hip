// thanos_factor: damping, diagonal extraction and the upper factor U of the inverse of the
// damped Hessian, H_d^{-1} = U^T U.
//
// Why one factor is enough.  Alg. 1 of the paper re-inverts the residual Hessian
// H_d[j:, j:] after every block (O(b^4/B), App. G.6).  With V upper triangular and
// H_d = V V^T, the trailing sub-matrix is H_d[j:, j:] = V[j:, j:] V[j:, j:]^T, so with
// U = V^{-1} (also upper triangular) inv(H_d[j:, j:]) = U[j:, j:]^T U[j:, j:] for every j.
//
// How U is computed.  Reversing the index order turns H_d = V V^T into an ordinary Cholesky
// factorisation: with J the reversal, A' = J H_d J = L L^T (L lower), V = J L J and
// U = J L^{-1} J.  So: (1) reversed, zero/identity-padded copy A' (ld = bp, a multiple of the
// factor block NB = 128); (2) right-looking blocked Cholesky: diagonal block in one workgroup
// (which also produces the inverse of the diagonal block), panel = product with that inverse,
// trailing update on the matrix cores, two-level (rank NB inside an outer block of 4 factor
// blocks, rank 4 NB for everything right of it); (3) L^{-1} by recursive doubling over
// block pairs, X21 = -Linv22 * (L21 * Linv11), two products per level; (4) U = J L^{-1} J.
// Everything is fp32.
#include <algorithm>

#include "gemm_tile.h"

namespace thanos {

constexpr int NB = kFactorNB;

// ------------------------------------------------------------------------------------------
// xnorm2[j] = H[j][j];  lam = damping * mean_j H[j][j]  (sum in fp64, fixed order).
// One workgroup of 1024 threads.
__global__ __launch_bounds__(1024) void k_diag_stats(const float* __restrict__ H, int64_t b,
                                                     float damping, float* __restrict__ xnorm2,
                                                     float* __restrict__ lam_out,
                                                     int32_t* __restrict__ info) {
  __shared__ double part[1024];
  double s = 0.0;
  for (int64_t j = threadIdx.x; j < b; j += 1024) {
    const float d = H[j * b + j];
    xnorm2[j] = d;
    s += (double)d;
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *lam_out = (float)((double)damping * (part[0] / (double)b));
    *info = 0;
  }
}

// A'[i][j] = H_d[b-1-i][b-1-j] for i >= j (read from the lower triangle of H as
// H[b-1-j][b-1-i]); identity on the padding; zero above the diagonal.  32x32 tiles through
// LDS so that both the read of H and the write of A' are coalesced.
__global__ __launch_bounds__(256) void k_reverse_pad(const float* __restrict__ H, int64_t b,
                                                     const float* __restrict__ lam_p,
                                                     float* __restrict__ Ap, int64_t bp) {
  __shared__ float t[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  const int64_t i0 = (int64_t)blockIdx.y * 32, j0 = (int64_t)blockIdx.x * 32;
  if (j0 > i0 + 31) {  // tile entirely above the diagonal
    for (int r = ty; r < 32; r += 8) Ap[(i0 + r) * bp + j0 + tx] = 0.f;
    return;
  }
  // A'[i0+r][j0+cidx] = H[b-1-(j0+cidx)][b-1-(i0+r)]: source rows are indexed by cidx,
  // source columns by r.  Load with lanes along r (source columns, contiguous, descending).
  for (int cc = ty; cc < 32; cc += 8) {
    const int64_t sr = b - 1 - (j0 + cc);
    const int64_t sc = b - 1 - (i0 + tx);
    float v = 0.f;
    if (sr >= 0 && sc >= 0 && sr < b && sc < b && sr >= sc) v = H[sr * b + sc];
    t[cc][tx] = v;  // t[cidx][r]
  }
  __syncthreads();
  const float lam = *lam_p;
  for (int r = ty; r < 32; r += 8) {
    const int64_t i = i0 + r, j = j0 + tx;
    float v;
    if (j > i) v = 0.f;
    else if (i >= b) v = (i == j) ? 1.f : 0.f;
    else v = t[tx][r] + ((i == j) ? lam : 0.f);
    Ap[i * bp + j] = v;
  }
}

// ------------------------------------------------------------------------------------------
// Cholesky factor and inverse of one NB x NB diagonal block, one workgroup of 256 threads.
//   in : lower triangle of A'[kb*NB .. , kb*NB ..]
//   out: L_kk in the same place (lower triangle), Linv diagonal block = L_kk^{-1} (full
//        square, zeros above the diagonal).
//
// In-place elimination on one array X held in REGISTERS, 8x8 elements per thread (thread
// (bi, bj) owns rows 8bi.., columns 8bj..).  Before step k column j > k of X holds the
// partially reduced A, afterwards (j <= k) it holds column j of the growing inverse T:
//   l_i = X[i][k] / sqrt(d),  d = X[k][k]
//   X[i][j] -= l_i * X[j][k]/sqrt(d)   (j > k: Cholesky update, symmetric source)
//   X[i][j] -= l_i * X[k][j]/sqrt(d)   (j < k: the same row operation applied to T)
//   X[i][k]  = -l_i / sqrt(d),  X[k][j<k] /= sqrt(d),  X[k][k] = 1/sqrt(d)
// for rows i > k only.  Per step the owners of column k and of row k publish 128 values
// through a double-buffered LDS vector (one barrier per step); everything else is register
// arithmetic with static indices (the 8 steps of a block column are unrolled).
__global__ __launch_bounds__(256) void k_chol_diag(float* __restrict__ Ap, float* __restrict__ Linv,
                                                   int64_t bp, int kb_glob, int64_t b,
                                                   int32_t* __restrict__ info) {
  __shared__ __attribute__((aligned(16))) float buf[2][NB];
  __shared__ float Lout[NB][NB + 1];
  const int tid = threadIdx.x;
  const int bi = tid >> 4, bj = tid & 15;
  float* A = Ap + ((int64_t)kb_glob * NB) * bp + (int64_t)kb_glob * NB;
  float* Li = Linv + ((int64_t)kb_glob * NB) * bp + (int64_t)kb_glob * NB;
  float X[8][8];
#pragma unroll
  for (int ii = 0; ii < 8; ++ii) {
    const float4 a0 = *reinterpret_cast<const float4*>(A + (int64_t)(8 * bi + ii) * bp + 8 * bj);
    const float4 a1 = *reinterpret_cast<const float4*>(A + (int64_t)(8 * bi + ii) * bp + 8 * bj + 4);
    X[ii][0] = a0.x; X[ii][1] = a0.y; X[ii][2] = a0.z; X[ii][3] = a0.w;
    X[ii][4] = a1.x; X[ii][5] = a1.y; X[ii][6] = a1.z; X[ii][7] = a1.w;
  }
  int badk = -1;
  for (int kb = 0; kb < NB / 8; ++kb) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int k = 8 * kb + kk;
      float* bw = buf[k & 1];
      // publish column k (rows >= k) and row k (columns < k): 8 consecutive entries per owner
      if (bj == kb && bi == kb) {
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (e < kk) ? X[kk][e] : X[e][kk];
        *reinterpret_cast<float4*>(&bw[8 * kb]) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(&bw[8 * kb + 4]) = make_float4(v[4], v[5], v[6], v[7]);
      } else if (bj == kb && bi > kb) {
        *reinterpret_cast<float4*>(&bw[8 * bi]) =
            make_float4(X[0][kk], X[1][kk], X[2][kk], X[3][kk]);
        *reinterpret_cast<float4*>(&bw[8 * bi + 4]) =
            make_float4(X[4][kk], X[5][kk], X[6][kk], X[7][kk]);
      } else if (bi == kb && bj < kb) {
        *reinterpret_cast<float4*>(&bw[8 * bj]) =
            make_float4(X[kk][0], X[kk][1], X[kk][2], X[kk][3]);
        *reinterpret_cast<float4*>(&bw[8 * bj + 4]) =
            make_float4(X[kk][4], X[kk][5], X[kk][6], X[kk][7]);
      }
      __syncthreads();
      float d = bw[k];
      if (!(d > 0.f)) {
        if (badk < 0) badk = k;
        d = 1.f;
      }
      const float sd = sqrtf(d);
      const float inv = 1.f / sd;
      if (bi >= kb) {  // rows of earlier block rows are final
        const float4 r0 = *reinterpret_cast<const float4*>(&bw[8 * bi]);
        const float4 r1 = *reinterpret_cast<const float4*>(&bw[8 * bi + 4]);
        const float4 c0 = *reinterpret_cast<const float4*>(&bw[8 * bj]);
        const float4 c1 = *reinterpret_cast<const float4*>(&bw[8 * bj + 4]);
        float li[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
        float vj[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        const float s_hi = (bi > kb) ? inv : 0.f;  // rows of this thread with row <= k get 0
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          li[e] *= (e > kk) ? inv : s_hi;
          vj[e] *= inv;
        }
        if (bi == kb) {  // row k becomes final: T[k][j<k] scaled, T[k][k] = 1/sqrt(d)
          if (bj < kb) {
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) X[kk][jj] = vj[jj];
          } else if (bj == kb) {
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
              if (jj < kk) X[kk][jj] = vj[jj];
              else if (jj == kk) X[kk][jj] = inv;
            }
          }
        }
#pragma unroll
        for (int ii = 0; ii < 8; ++ii)
#pragma unroll
          for (int jj = 0; jj < 8; ++jj) X[ii][jj] = fmaf(-li[ii], vj[jj], X[ii][jj]);
        if (bj == kb) {  // column k: publish L[:, k], start column k of the inverse
          if (bi > kb) {
#pragma unroll
            for (int ii = 0; ii < 8; ++ii) {
              Lout[8 * bi + ii][k] = li[ii];
              X[ii][kk] = -li[ii] * inv;
            }
          } else {
#pragma unroll
            for (int ii = 0; ii < 8; ++ii) {
              if (ii > kk) {
                Lout[8 * bi + ii][k] = li[ii];
                X[ii][kk] = -li[ii] * inv;
              } else if (ii == kk) {
                Lout[8 * bi + ii][k] = sd;
              }
            }
          }
        }
      }
    }
  }
  if (badk >= 0 && tid == 0) {
    const int64_t orig = b - ((int64_t)kb_glob * NB + badk);  // 1-based original column
    atomicCAS(info, 0, (int32_t)(orig > 0 ? orig : 1));
  }
  __syncthreads();
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e / NB, j = e % NB;
    if (j <= i) A[(int64_t)i * bp + j] = Lout[i][j];
  }
#pragma unroll
  for (int ii = 0; ii < 8; ++ii) {
    const int i = 8 * bi + ii;
    float o[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) o[jj] = (8 * bj + jj <= i) ? X[ii][jj] : 0.f;
    float* dst = Li + (int64_t)i * bp + 8 * bj;
    *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
    *reinterpret_cast<float4*>(dst + 4) = make_float4(o[4], o[5], o[6], o[7]);
  }
}

// ------------------------------------------------------------------------------------------
// Inverse of the block lower-triangular L by recursive doubling.  At level S (in blocks) the
// matrix is cut into pairs of S-block halves; for each pair
//     Tbuf21 = L21 * Linv11        (Linv11 lower triangular: k-blocks >= column block)
//     Linv21 = -Linv22 * Tbuf21    (Linv22 lower triangular: k-blocks <= row block)
struct TrinvArgs {
  const float* L;
  float* Linv;
  float* T;
  int64_t bp;
  int nb, S;
};

__global__ __launch_bounds__(256) void k_trinv_T(TrinvArgs a) {
  __shared__ GemmSmem sm;
  const int tj = blockIdx.x, ti = blockIdx.y, p = blockIdx.z;
  const int base = 2 * p * a.S;
  const int gi = base + a.S + ti, gj = base + tj;
  if (gi >= a.nb) return;
  const float* A = a.L + ((int64_t)gi * NB) * a.bp + (int64_t)base * NB;   // [m][k]
  const float* B = a.Linv + ((int64_t)base * NB) * a.bp + (int64_t)gj * NB;  // [k][n]
  TileAcc acc;
  acc_zero(acc);
  gemm_tile<false, true>(acc, sm, A, a.bp, NB, B, a.bp, NB, tj * NB, a.S * NB, true, true);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
  float* C = a.T + ((int64_t)gi * NB) * a.bp + (int64_t)gj * NB;
#pragma unroll
  for (int f = 0; f < 2; ++f)
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        C[(int64_t)acc_row(wm, f, r, lane) * a.bp + acc_col(wn, g, lane)] = acc.v[f][g][r];
}

__global__ __launch_bounds__(256) void k_trinv_X(TrinvArgs a) {
  __shared__ GemmSmem sm;
  const int tj = blockIdx.x, ti = blockIdx.y, p = blockIdx.z;
  const int base = 2 * p * a.S;
  const int gi = base + a.S + ti, gj = base + tj;
  if (gi >= a.nb) return;
  const float* A = a.Linv + ((int64_t)gi * NB) * a.bp + (int64_t)(base + a.S) * NB;  // [m][k]
  const float* B = a.T + ((int64_t)(base + a.S) * NB) * a.bp + (int64_t)gj * NB;     // [k][n]
  TileAcc acc;
  acc_zero(acc);
  gemm_tile<false, true>(acc, sm, A, a.bp, NB, B, a.bp, NB, 0, (ti + 1) * NB, true, true);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
  float* C = a.Linv + ((int64_t)gi * NB) * a.bp + (int64_t)gj * NB;
#pragma unroll
  for (int f = 0; f < 2; ++f)
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        C[(int64_t)acc_row(wm, f, r, lane) * a.bp + acc_col(wn, g, lane)] = -acc.v[f][g][r];
}

// U[i][j] = Linv[b-1-i][b-1-j] for j >= i, else 0.
__global__ __launch_bounds__(256) void k_reverse_out(const float* __restrict__ Linv, int64_t bp,
                                                     float* __restrict__ U, int64_t b) {
  const int64_t i = blockIdx.y;
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= b) return;
  U[i * b + j] = (j >= i) ? Linv[(b - 1 - i) * bp + (b - 1 - j)] : 0.f;
}

static inline int64_t padded(int64_t b) { return ceil_div(b, NB) * NB; }

size_t factor_workspace_bytes(int64_t b) {
  const int64_t bp = padded(b);
  return 3 * (size_t)bp * bp * sizeof(float) + 256;
}

thanos_status factor(hipStream_t s, const float* H, int64_t b, float damping, float* U,
                     float* xnorm2, void* ws, int32_t* info) {
  const int64_t bp = padded(b);
  const int nb = (int)(bp / NB);
  float* lam = reinterpret_cast<float*>(ws);
  float* Ap = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + 256);
  float* Linv = Ap + bp * bp;
  float* Tb = Linv + bp * bp;

  hipLaunchKernelGGL(k_diag_stats, dim3(1), dim3(1024), 0, s, H, b, damping, xnorm2, lam, info);
  THANOS_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_reverse_pad, dim3((unsigned)(bp / 32), (unsigned)(bp / 32)), dim3(256), 0,
                     s, H, b, lam, Ap, bp);
  THANOS_LAUNCH_CHECK();

  // Two-level blocking: inside an outer block of kOuter factor blocks the trailing update of a
  // step only reaches the columns of that outer block (narrow, K = NB); everything to the right
  // gets one update per outer block with K = kOuter*NB, which reads and writes the trailing
  // matrix kOuter times less often and runs the matrix cores on long reductions.
  // That wide update is split in two: the column strip of the NEXT outer block stays on the
  // caller's stream (the next diagonal block needs it), the rest runs on a second stream next
  // to the latency-bound diagonal / panel chain of the next outer block.  Column ranges of the
  // two streams are disjoint until the next strip, which waits for the previous rest.
  constexpr int kOuter = 4;
  const int n_outer = (nb + kOuter - 1) / kOuter;
  AuxStream aux(2 * n_outer);
  if (!aux.ok) return THANOS_ERR_HIP;
  int pending_join = -1;  // event index recorded on the aux stream after the last "rest"
  for (int k = 0; k < nb; ++k) {
    hipLaunchKernelGGL(k_chol_diag, dim3(1), dim3(256), 0, s, Ap, Linv, bp, k, b, info);
    THANOS_LAUNCH_CHECK();
    const int64_t rem = bp - (int64_t)(k + 1) * NB;
    if (rem <= 0) break;
    float* panel = Ap + ((int64_t)(k + 1) * NB) * bp + (int64_t)k * NB;
    const float* dinv = Linv + ((int64_t)k * NB) * bp + (int64_t)k * NB;
    // L_ik = A_ik * Linv_kk^T  (in place, all rows below the diagonal block)
    thanos_status st = gemm_f32(s, false, false, rem, NB, NB, 1.f, panel, bp, dinv, bp, 0.f,
                                panel, bp, false);
    if (st != THANOS_OK) return st;
    const int ob = k / kOuter;
    const int ob_begin = ob * kOuter;
    const int ob_end = std::min(nb, ob_begin + kOuter);
    // narrow: A_ij -= L_ik L_jk^T for block columns k < j < ob_end, lower tiles
    const int64_t ncols = (int64_t)(ob_end - (k + 1)) * NB;
    if (ncols > 0) {
      float* trail = Ap + ((int64_t)(k + 1) * NB) * bp + (int64_t)(k + 1) * NB;
      st = gemm_f32(s, false, false, rem, ncols, NB, -1.f, panel, bp, panel, bp, 1.f, trail, bp,
                    true);
      if (st != THANOS_OK) return st;
    }
    // wide: after the last step of an outer block, everything right of it
    if (k + 1 == ob_end && ob_end < nb) {
      const int next_end = std::min(nb, ob_end + kOuter);
      const int64_t kk = (int64_t)(ob_end - ob_begin) * NB;
      const float* lp = Ap + ((int64_t)ob_end * NB) * bp + (int64_t)ob_begin * NB;
      // fork: the rest (rows and columns >= next_end) on the second stream
      if (next_end < nb) {
        THANOS_HIP_CHECK(hipEventRecord(aux.ev[2 * ob], s));
        THANOS_HIP_CHECK(hipStreamWaitEvent(aux.stream, aux.ev[2 * ob], 0));
        const int64_t rest = bp - (int64_t)next_end * NB;
        const float* lr = lp + ((int64_t)(next_end - ob_end) * NB) * bp;
        float* cr = Ap + ((int64_t)next_end * NB) * bp + (int64_t)next_end * NB;
        st = gemm_f32(aux.stream, false, false, rest, rest, kk, -1.f, lr, bp, lr, bp, 1.f, cr, bp,
                      true);
        if (st != THANOS_OK) return st;
      }
      // the strip of the next outer block: it was last written by the previous rest
      if (pending_join >= 0) THANOS_HIP_CHECK(hipStreamWaitEvent(s, aux.ev[pending_join], 0));
      {
        const int64_t rows = bp - (int64_t)ob_end * NB;
        const int64_t cols = (int64_t)(next_end - ob_end) * NB;
        float* cs = Ap + ((int64_t)ob_end * NB) * bp + (int64_t)ob_end * NB;
        st = gemm_f32(s, false, false, rows, cols, kk, -1.f, lp, bp, lp, bp, 1.f, cs, bp, true);
        if (st != THANOS_OK) return st;
      }
      if (next_end < nb) {
        THANOS_HIP_CHECK(hipEventRecord(aux.ev[2 * ob + 1], aux.stream));
        pending_join = 2 * ob + 1;
      }
    }
  }
  if (pending_join >= 0) THANOS_HIP_CHECK(hipStreamWaitEvent(s, aux.ev[pending_join], 0));

  for (int S = 1; S < nb; S *= 2) {
    TrinvArgs a{Ap, Linv, Tb, bp, nb, S};
    dim3 grid((unsigned)S, (unsigned)S, (unsigned)ceil_div(nb, 2 * S));
    hipLaunchKernelGGL(k_trinv_T, grid, dim3(256), 0, s, a);
    THANOS_LAUNCH_CHECK();
    hipLaunchKernelGGL(k_trinv_X, grid, dim3(256), 0, s, a);
    THANOS_LAUNCH_CHECK();
  }

  hipLaunchKernelGGL(k_reverse_out, dim3((unsigned)ceil_div(b, 256), (unsigned)b), dim3(256), 0, s,
                     Linv, bp, U, b);
  THANOS_LAUNCH_CHECK();
  return THANOS_OK;
}

}  // namespace thanos
