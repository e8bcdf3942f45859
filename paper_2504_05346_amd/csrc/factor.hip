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

#include "gemm_tile_x3.h"

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
// Cholesky factor and inverse of one NB x NB diagonal block, one workgroup of 4 wavefronts.
//   in : lower triangle of A'[kb*NB .. , kb*NB ..]
//   out: L_kk in the same place (lower triangle), Linv diagonal block = L_kk^{-1} (full
//        square, zeros above the diagonal).
//
// The block lives in LDS (S: A -> L, T: the inverse) and is processed in four steps of 32
// columns.  Everything runs on the matrix cores, including the pivot loop:
//
//  * Pivot loop of step j (32 pivots, no barrier).  A 32x32 tile held in the accumulator
//    layout of v_mfma_f32_32x32x2_f32 has row k in lanes (lo = column, hi = hk) of register rk.
//    For a symmetric tile D that row is also column k, i.e. it is already laid out as BOTH
//    operands of the rank-1 update D -= u u^T / d, u = D[k][:], d = u_k: one MFMA per pivot,
//    no cross-lane traffic except the broadcast of d.  Column k of L is u / sqrt(d).
//    Every wavefront keeps its own copy of the diagonal tile D and repeats that update, so
//    that it can apply the same pivot to a second tile without talking to the others:
//      wavefront 0     : T~ (starts as I), T~ -= (u/d) T~[k][:] for rows != k; after 32 pivots
//                        T~ = L~^{-1} (unit lower), and L_jj^{-1} = diag(1/sqrt(d)) T~;
//      wavefront w >= 1: the panel tile A_ij (i = j + w) held TRANSPOSED, so that its column k
//                        is again row k of the register tile: A_ij^T -= u (A_ij[:,k] / d)^T;
//                        column k of L_ij is A_ij[:,k] / sqrt(d).
//  * Trailing update of the remaining lower tiles, A_il -= L_ij L_lj^T (i >= l > j), operands
//    read from LDS.
//  * After the four steps: the off-diagonal blocks of the inverse by recursive doubling over
//    32- and 64-blocks, X21 = -T22 (L21 T11), with the strict upper tiles of S as scratch.
constexpr int kCdLd = NB + 1;  // LDS row stride in floats: conflict-free rows and columns
// S: the block (lower triangle = L in the end, strict upper 32-tiles = scratch and, later, the
// off-diagonal tiles (1,0) and (3,2) of the inverse); Td: the four diagonal 32x32 tiles of the
// inverse side by side (32 rows); 128 floats of scratch per wavefront.  85 KB: the kernel fits
// next to one workgroup of the matrix-product kernels on a compute unit instead of waiting for
// a whole unit to drain.
constexpr size_t kCholDiagSmem = ((size_t)(NB + 32) * kCdLd + 4 * 128) * sizeof(float);

__device__ __forceinline__ int cd_row(int r, int hi) { return 8 * (r >> 2) + 4 * hi + (r & 3); }

// acc += sign * A[0:32, 0:32] * B, A[m][k] at pa[m*kCdLd + k];
// B_KN: B[k][n] at pb[k*kCdLd + n], else B given as rows of n: B[k][n] at pb[n*kCdLd + k].
// All 32 operand values of a lane are fetched before the first MFMA.
template <bool B_KN>
__device__ __forceinline__ void cd_tile_mma32(f32x16& acc, const float* pa, const float* pb,
                                              float sign, int lo, int hi) {
  float av[16], bv[16];
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    av[q] = pa[lo * kCdLd + 2 * q + hi];
    bv[q] = B_KN ? pb[(2 * q + hi) * kCdLd + lo] : pb[lo * kCdLd + 2 * q + hi];
  }
#pragma unroll
  for (int q = 0; q < 16; ++q)
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(sign * av[q], bv[q], acc, 0, 0, 0);
}
__device__ __forceinline__ void cd_tile_load(f32x16& acc, const float* p, int lo, int hi) {
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = p[cd_row(r, hi) * kCdLd + lo];
}
__device__ __forceinline__ void cd_tile_store(float* p, const f32x16& acc, float scale, int lo,
                                              int hi) {
#pragma unroll
  for (int r = 0; r < 16; ++r) p[cd_row(r, hi) * kCdLd + lo] = scale * acc[r];
}

// The 32 pivots of one step for one wavefront.  ROLE 0: second tile is T~ (inverse of the
// diagonal tile), ROLE 1: second tile is the transposed panel tile whose rows in S start at
// `prow`.  `aux` points at this wavefront's 128 floats of LDS scratch.  Returns the first
// non-positive pivot (or -1).
//
// A wavefront cannot overlap its own vector instructions with its own MFMAs, so the pivot loop
// is kept to the bare chain: broadcast d, 1/d, the two operands, two MFMAs, one LDS write of
// the UNSCALED column of L.  The scaling by 1/sqrt(d) is applied to the whole tile afterwards.
template <int ROLE>
__device__ __forceinline__ int cd_pivots(float* S, float* T, float* aux, int c0, int prow, int lo,
                                         int hi) {
  f32x16 D, E;
  cd_tile_load(D, S + c0 * kCdLd + c0, lo, hi);
  if (ROLE == 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) E[r] = (cd_row(r, hi) == lo) ? 1.f : 0.f;
  } else {  // E[n][m] = A_ij[m][n]
#pragma unroll
    for (int r = 0; r < 16; ++r) E[r] = S[(prow + lo) * kCdLd + c0 + cd_row(r, hi)];
  }
  __syncthreads();  // every wavefront has its copy of D before L_jj overwrites it
  float* ltile = S + (ROLE == 0 ? c0 : prow) * kCdLd + c0;  // the tile of L this wavefront writes
  // key[h] = lo in the lanes that hold rows of half h (rows 4..7 mod 8 for h = 1), else -1:
  // (key[hk] >= k) selects the lanes of row k with column >= k, (key[hk] >= 0) all of row k.
  const int key[2] = {hi == 0 ? lo : -1, hi == 1 ? lo : -1};
  // where column k of L goes: lane lo owns row lo of the tile; the other half writes to scratch
  float* dst[2] = {hi == 0 ? ltile + lo * kCdLd : aux + 32 + lo,
                   hi == 1 ? ltile + lo * kCdLd : aux + 32 + lo};
  float dl = 1.f;  // pivot of column lo
#pragma unroll
  for (int k = 0; k < 32; ++k) {
    const int rk = 4 * (k >> 3) + (k & 3), hk = (k >> 2) & 1;
    const float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(D[rk]), k + 32 * hk));
    const float rd = __builtin_amdgcn_rcpf(d);
    const float u = (key[hk] >= k) ? D[rk] : 0.f;  // row k = column k of the reduced tile
    const float au = -rd * u;
    D = __builtin_amdgcn_mfma_f32_32x32x2f32(au, u, D, 0, 0, 0);
    dl = (lo == k) ? d : dl;
    const float ek = (key[hk] >= 0) ? E[rk] : 0.f;  // ROLE 0: T~[k][:], ROLE 1: A_ij[:, k]
    if (ROLE == 0) {
      const float a2 = (lo == k) ? 0.f : au;  // row k itself stays
      dst[hk][k] = u;                         // L_jj[:, k] * sqrt(d)
      E = __builtin_amdgcn_mfma_f32_32x32x2f32(a2, ek, E, 0, 0, 0);
    } else {
      dst[hk][k] = ek;                        // L_ij[:, k] * sqrt(d)
      E = __builtin_amdgcn_mfma_f32_32x32x2f32(u, -rd * ek, E, 0, 0, 0);
    }
  }
  // a non-positive pivot: report the first one (what was computed after it is garbage)
  const unsigned long long badm = __ballot(!(dl > 0.f)) & 0xffffffffull;
  const int bad = badm ? c0 + (__ffsll((long long)badm) - 1) : -1;
  float isd = __builtin_amdgcn_rsqf(dl);
  isd = fmaf(0.5f * isd, fmaf(-dl * isd, isd, 1.f), isd);
  // columns of L: scale column lo by 1/sqrt(d_lo)
  {
    f32x16 C;
    cd_tile_load(C, ltile, lo, hi);
    cd_tile_store(ltile, C, isd, lo, hi);
  }
  if (ROLE == 0) {  // L_jj^{-1} = diag(1/sqrt(d)) T~
    aux[lo] = isd;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      T[cd_row(r, hi) * kCdLd + c0 + lo] = E[r] * aux[cd_row(r, hi)];  // diagonal tile strip
  }
  return bad;
}

// Two wavefronts per SIMD at most: keeps the register budget at 256 so that the MFMA
// accumulators stay in ordinary vector registers (they are read lane-wise every pivot).
__global__ __launch_bounds__(256, 2) void k_chol_diag(float* __restrict__ Ap,
                                                      float* __restrict__ Linv, int64_t bp,
                                                      int kb_glob, int64_t b,
                                                      int32_t* __restrict__ info) {
  extern __shared__ __attribute__((aligned(16))) float cd_smem[];
  float* S = cd_smem;
  float* T = cd_smem + NB * kCdLd;  // Td: tile j of the inverse's diagonal at T + 32 j
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  float* aux = cd_smem + (NB + 32) * kCdLd + 128 * wave;  // per-wavefront scratch
  const int lo = lane & 31, hi = lane >> 5;
  float* A = Ap + ((int64_t)kb_glob * NB) * bp + (int64_t)kb_glob * NB;
  float* Li = Linv + ((int64_t)kb_glob * NB) * bp + (int64_t)kb_glob * NB;

  // lower triangle -> S, mirrored inside the diagonal 32x32 tiles (the pivot loop wants them
  // symmetric); the strict upper 32-tiles stay undefined (scratch).  The first 32 columns are
  // stored right away; the loads of the other 96 columns are issued now and stored to LDS after
  // the first pivot loop, which does not touch them.
  auto put = [&](int i, int c4, const float4& v) {
    const float vv[4] = {v.x, v.y, v.z, v.w};
    if (c4 <= i) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int j = c4 + t;
        if (j <= i) {
          S[i * kCdLd + j] = vv[t];
          if ((j >> 5) == (i >> 5)) S[j * kCdLd + i] = vv[t];
        }
      }
    }
  };
  constexpr int kVecA = NB * 8 / 256, kVecB = NB * 24 / 256;
  float4 va[kVecA], vb[kVecB];
#pragma unroll
  for (int q = 0; q < kVecA; ++q) {
    const int e = tid + 256 * q, i = e / 8, c4 = (e % 8) * 4;
    va[q] = (c4 <= i) ? *reinterpret_cast<const float4*>(A + (int64_t)i * bp + c4)
                      : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int q = 0; q < kVecB; ++q) {
    const int e = tid + 256 * q, i = e / 24, c4 = 32 + (e % 24) * 4;
    vb[q] = (c4 <= i) ? *reinterpret_cast<const float4*>(A + (int64_t)i * bp + c4)
                      : make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int q = 0; q < kVecA; ++q) {
    const int e = tid + 256 * q;
    put(e / 8, (e % 8) * 4, va[q]);
  }
  __syncthreads();

  int badk = -1;
  for (int j = 0; j < NB / 32; ++j) {
    const int c0 = 32 * j;
    const int ti = j + wave;  // panel tile row of wavefronts >= 1
    if (wave == 0) {
      const int bad = cd_pivots<0>(S, T, aux, c0, 0, lo, hi);
      if (badk < 0) badk = bad;
    } else if (ti < NB / 32) {
      (void)cd_pivots<1>(S, T, aux, c0, 32 * ti, lo, hi);
    } else {
      __syncthreads();  // the barrier inside cd_pivots
    }
    if (j == 0) {
#pragma unroll
      for (int q = 0; q < kVecB; ++q) {
        const int e = tid + 256 * q;
        put(e / 24, 32 + (e % 24) * 4, vb[q]);
      }
    }
    __syncthreads();
    // trailing tiles (i, l), j < l <= i < 4, dealt round-robin to the wavefronts
    {
      int t = 0;
      for (int i = j + 1; i < NB / 32; ++i)
        for (int l = j + 1; l <= i; ++l, ++t) {
          if ((t & 3) != wave) continue;
          f32x16 C;
          float* pc = S + (32 * i) * kCdLd + 32 * l;
          cd_tile_load(C, pc, lo, hi);
          cd_tile_mma32<false>(C, S + (32 * i) * kCdLd + c0, S + (32 * l) * kCdLd + c0, -1.f, lo,
                               hi);
          cd_tile_store(pc, C, 1.f, lo, hi);
        }
    }
    __syncthreads();
  }
  if (badk >= 0 && tid == 0) {
    const int64_t orig = b - ((int64_t)kb_glob * NB + badk);  // 1-based original column
    atomicCAS(info, 0, (int32_t)(orig > 0 ? orig : 1));
  }

  // inverse, 32 -> 64: pairs (0,1) and (2,3).  W = L21 T11 goes to the strict upper tile
  // (p, p+1) of S and is then replaced, in place, by T21 = -T22 W (one wavefront, all operands
  // are in registers before the result is stored).
  if (wave < 2) {
    const int p0 = 64 * wave, p1 = p0 + 32;
    f32x16 C;
#pragma unroll
    for (int r = 0; r < 16; ++r) C[r] = 0.f;
    cd_tile_mma32<true>(C, S + p1 * kCdLd + p0, T + p0, 1.f, lo, hi);
    float* w = S + p0 * kCdLd + p1;
    cd_tile_store(w, C, 1.f, lo, hi);
#pragma unroll
    for (int r = 0; r < 16; ++r) C[r] = 0.f;
    cd_tile_mma32<true>(C, T + p1, w, 1.f, lo, hi);
    cd_tile_store(w, C, -1.f, lo, hi);  // tile (1,0) of the inverse at S[0:32, 32:64], (3,2) at S[64:96, 96:128]
  }
  __syncthreads();
  // 64 -> 128: W = L[64:128, 0:64] T[0:64, 0:64] into S[0:64, 64:128], then
  // T[64:128, 0:64] = -T[64:128, 64:128] W straight to global memory; one 32x32 tile per
  // wavefront.  Tile (a, b) of a 64x64 block of the inverse: diagonal ones in the strip, the
  // off-diagonal one in S as stored above.
  {
    const int ti = wave >> 1, tj = wave & 1;  // tile inside the 64x64 block
    f32x16 C;
#pragma unroll
    for (int r = 0; r < 16; ++r) C[r] = 0.f;
    // T[0:64,0:64] is lower triangular: 32-blocks of k from tj
    for (int kb = tj; kb < 2; ++kb) {
      const float* t11 = (kb == tj) ? T + 32 * kb : S + 32;  // tile (kb, tj) of T[0:64, 0:64]
      cd_tile_mma32<true>(C, S + (64 + 32 * ti) * kCdLd + 32 * kb, t11, 1.f, lo, hi);
    }
    cd_tile_store(S + (32 * ti) * kCdLd + 64 + 32 * tj, C, 1.f, lo, hi);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) C[r] = 0.f;
    // T[64:128,64:128] is lower triangular: 32-blocks of k up to ti
    for (int kb = 0; kb <= ti; ++kb) {
      const float* t22 = (kb == ti) ? T + 64 + 32 * kb : S + 64 * kCdLd + 96;  // tile (ti, kb)
      cd_tile_mma32<true>(C, t22, S + (32 * kb) * kCdLd + 64 + 32 * tj, 1.f, lo, hi);
    }
    float* g = Li + (int64_t)(64 + 32 * ti) * bp + 32 * tj;
#pragma unroll
    for (int r = 0; r < 16; ++r) g[(int64_t)cd_row(r, hi) * bp + lo] = -C[r];
  }
  __syncthreads();
  {
    constexpr int kVec = NB * (NB / 4) / 256;
    float4 l[kVec], t[kVec];
#pragma unroll
    for (int q = 0; q < kVec; ++q) {
      const int e = tid + 256 * q, i = e / (NB / 4), c4 = (e % (NB / 4)) * 4;
      float lv[4], tv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int cc = c4 + u;
        const bool low = cc <= i;
        lv[u] = low ? S[i * kCdLd + cc] : 0.f;
        // inverse: diagonal tiles from the strip, tiles (1,0) and (3,2) from the upper tiles of S
        // (the lower left 64x64 quadrant is in global memory already and is skipped below)
        const float* tp = ((i >> 5) == (cc >> 5)) ? T + (i & 31) * kCdLd + cc
                                                  : S + (i - 32) * kCdLd + cc + 32;
        tv[u] = (low && !(i >= 64 && cc < 64)) ? *tp : 0.f;
      }
      l[q] = make_float4(lv[0], lv[1], lv[2], lv[3]);
      t[q] = make_float4(tv[0], tv[1], tv[2], tv[3]);
    }
#pragma unroll
    for (int q = 0; q < kVec; ++q) {
      const int e = tid + 256 * q, i = e / (NB / 4), c4 = (e % (NB / 4)) * 4;
      if (c4 + 3 <= i) {
        *reinterpret_cast<float4*>(A + (int64_t)i * bp + c4) = l[q];
      } else {
        const float lv[4] = {l[q].x, l[q].y, l[q].z, l[q].w};
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (c4 + u <= i) A[(int64_t)i * bp + c4 + u] = lv[u];
      }
      if (!(i >= 64 && c4 < 64)) *reinterpret_cast<float4*>(Li + (int64_t)i * bp + c4) = t[q];
    }
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
  int p0, c0;  // this launch: pairs from p0 (blockIdx.z), tile columns of a pair from c0 (blockIdx.x)
};

__global__ __launch_bounds__(kXThreads, 4) void k_trinv_T(TrinvArgs a) {
  extern __shared__ __attribute__((aligned(16))) char sm[];
  const int tj = a.c0 + blockIdx.x, ti = blockIdx.y, p = a.p0 + blockIdx.z;
  const int base = 2 * p * a.S;
  const int gi = base + a.S + ti, gj = base + tj;
  if (gi >= a.nb) return;
  const float* A = a.L + ((int64_t)gi * NB) * a.bp + (int64_t)base * NB;   // [m][k]
  const float* B = a.Linv + ((int64_t)base * NB) * a.bp + (int64_t)gj * NB;  // [k][n]
  TileAcc acc;
  acc_zero(acc);
  gemm_tile_x3<false, true>(acc, sm, A, a.bp, NB, B, a.bp, NB, tj * NB, a.S * NB, true, true);
  x3_write_tile(acc, sm, a.T + ((int64_t)gi * NB) * a.bp + (int64_t)gj * NB, a.bp, 1.f);
}

__global__ __launch_bounds__(kXThreads, 4) void k_trinv_X(TrinvArgs a) {
  extern __shared__ __attribute__((aligned(16))) char sm[];
  const int tj = a.c0 + blockIdx.x, ti = blockIdx.y, p = a.p0 + blockIdx.z;
  const int base = 2 * p * a.S;
  const int gi = base + a.S + ti, gj = base + tj;
  if (gi >= a.nb) return;
  const float* A = a.Linv + ((int64_t)gi * NB) * a.bp + (int64_t)(base + a.S) * NB;  // [m][k]
  const float* B = a.T + ((int64_t)(base + a.S) * NB) * a.bp + (int64_t)gj * NB;     // [k][n]
  TileAcc acc;
  acc_zero(acc);
  gemm_tile_x3<false, true>(acc, sm, A, a.bp, NB, B, a.bp, NB, 0, (ti + 1) * NB, true, true);
  x3_write_tile(acc, sm, a.Linv + ((int64_t)gi * NB) * a.bp + (int64_t)gj * NB, a.bp, -1.f);
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

const float* factor_L(const void* ws, int64_t b, int64_t* ld) {
  *ld = padded(b);
  return reinterpret_cast<const float*>(reinterpret_cast<const char*>(ws) + 256);
}

size_t factor_workspace_bytes(int64_t b) {
  const int64_t bp = padded(b);
  return 3 * (size_t)bp * bp * sizeof(float) + 256;
}

thanos_status factor(hipStream_t s, const float* H, int64_t b, float damping, float* U,
                     float* xnorm2, void* ws, int32_t* info, bool single_stream) {
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
  THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_chol_diag),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kCholDiagSmem));
  constexpr int kOuter = 4;
  const int n_outer = (nb + kOuter - 1) / kOuter;
  AuxStream aux(s, 2 * n_outer, single_stream);
  if (!aux.ok) return THANOS_ERR_HIP;

  // The inverse of L (recursive doubling, see k_trinv_T / k_trinv_X) does not wait for the end
  // of the factorisation: the merge of two halves at level S needs, for its first product
  // L21 * Linv11, only the column blocks of the FIRST half (final once their panels are
  // solved), and for its second product the inverse of the second half.  After every outer
  // block the merges that have become possible are queued on a third stream, lowest level
  // first and the first product before the second at each level (the order of their
  // dependencies); they fill the compute units that the chain of diagonal blocks leaves idle.
  // Regions written by different merges are disjoint, and none overlaps what the
  // factorisation still writes.
  THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_trinv_T),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kXSmemBytes));
  THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_trinv_X),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kXSmemBytes));
  AuxStream tri(s, n_outer + 1, single_stream);
  if (!tri.ok) return THANOS_ERR_HIP;
  int tri_done = -1;  // blocks 0..tri_done have been handed to the inversion
  int tri_batches = 0;
  constexpr int tri_cap = 512;  // workgroups of one launch while the factorisation runs (256 or
                                // 384 measured the same, 192 and fewer slower)
  auto trinv_upto = [&](int kdone) -> thanos_status {
    // blocks <= kdone: diagonal inverse known, panel below solved (recorded on s by the caller)
    THANOS_CHECK(tri.fork(tri_batches));
    ++tri_batches;
    for (int S = 1; S < nb; S *= 2) {
      for (int second = 0; second < 2; ++second) {
        int p_lo = -1, p_hi = -1;
        for (int p = 0; 2 * p * S + S < nb; ++p) {
          const int e = second ? std::min(2 * p * S + 2 * S, nb) - 1 : 2 * p * S + S - 1;
          if (e > tri_done && e <= kdone) {
            if (p_lo < 0) p_lo = p;
            p_hi = p;
          }
        }
        if (p_lo < 0) continue;
        const int np = p_hi - p_lo + 1;
        // rows of the second half that exist (the last pair of a level may be cut short)
        const int rows = std::min(S, nb - (2 * p_hi * S + S));
        const int rows_all = np > 1 ? S : rows;
        // while the factorisation runs, a launch takes at most tri_cap workgroups (one round of
        // the chip's workgroup slots), so that the short kernels of the chain are not queued
        // behind thousands of long-running tiles
        int cols = S;
        if (kdone != nb - 1) cols = std::max(1, std::min(S, tri_cap / (rows_all * np)));
        for (int c0 = 0; c0 < S; c0 += cols) {
          TrinvArgs a{Ap, Linv, Tb, bp, nb, S, p_lo, c0};
          dim3 grid((unsigned)std::min(cols, S - c0), (unsigned)rows_all, (unsigned)np);
          if (second)
            hipLaunchKernelGGL(k_trinv_X, grid, dim3(kXThreads), kXSmemBytes, tri.stream, a);
          else
            hipLaunchKernelGGL(k_trinv_T, grid, dim3(kXThreads), kXSmemBytes, tri.stream, a);
          THANOS_LAUNCH_CHECK();
        }
      }
    }
    tri_done = kdone;
    return THANOS_OK;
  };
  int pending_join = -1;  // event index recorded on the aux stream after the last "rest"
  for (int k = 0; k < nb; ++k) {
    hipLaunchKernelGGL(k_chol_diag, dim3(1), dim3(256), kCholDiagSmem, s, Ap, Linv, bp, k, b, info);
    THANOS_LAUNCH_CHECK();
    const int64_t rem = bp - (int64_t)(k + 1) * NB;
    if (rem <= 0) {
      thanos_status st = trinv_upto(k);
      if (st != THANOS_OK) return st;
      break;
    }
    float* panel = Ap + ((int64_t)(k + 1) * NB) * bp + (int64_t)k * NB;
    const float* dinv = Linv + ((int64_t)k * NB) * bp + (int64_t)k * NB;
    // L_ik = A_ik * Linv_kk^T  (in place, all rows below the diagonal block)
    thanos_status st = gemm_f32(s, false, false, rem, NB, NB, 1.f, panel, bp, dinv, bp, 0.f,
                                panel, bp, false);
    if (st != THANOS_OK) return st;
    if ((k + 1) % kOuter == 0) {
      st = trinv_upto(k);
      if (st != THANOS_OK) return st;
    }
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
      // The strip of the next outer block first: it is on the critical path (the next diagonal
      // block waits for it) and gets the chip to itself for the ~25 us it needs; launched behind
      // the rest, it shared the compute units with that much larger product and took 80-100 us.
      // It was last written by the previous rest.
      if (pending_join >= 0) THANOS_CHECK(aux.join(pending_join));
      {
        const int64_t rows = bp - (int64_t)ob_end * NB;
        const int64_t cols = (int64_t)(next_end - ob_end) * NB;
        float* cs = Ap + ((int64_t)ob_end * NB) * bp + (int64_t)ob_end * NB;
        st = gemm_f32(s, false, false, rows, cols, kk, -1.f, lp, bp, lp, bp, 1.f, cs, bp, true);
        if (st != THANOS_OK) return st;
      }
      // fork: the rest (rows and columns >= next_end) on the second stream, next to the
      // latency-bound chain of the next outer block (the fork point lies behind the strip, which
      // costs the rest nothing: the two write disjoint columns)
      if (next_end < nb) {
        THANOS_CHECK(aux.fork(2 * ob));
        const int64_t rest = bp - (int64_t)next_end * NB;
        const float* lr = lp + ((int64_t)(next_end - ob_end) * NB) * bp;
        float* cr = Ap + ((int64_t)next_end * NB) * bp + (int64_t)next_end * NB;
        st = gemm_f32(aux.stream, false, false, rest, rest, kk, -1.f, lr, bp, lr, bp, 1.f, cr, bp,
                      true);
        if (st != THANOS_OK) return st;
        THANOS_CHECK(aux.record(2 * ob + 1));
        pending_join = 2 * ob + 1;
      }
    }
  }
  if (pending_join >= 0) THANOS_CHECK(aux.join(pending_join));

  THANOS_CHECK(tri.record(n_outer));
  THANOS_CHECK(tri.join(n_outer));

  hipLaunchKernelGGL(k_reverse_out, dim3((unsigned)ceil_div(b, 256), (unsigned)b), dim3(256), 0, s,
                     Linv, bp, U, b);
  THANOS_LAUNCH_CHECK();
  return THANOS_OK;
}

}  // namespace thanos
