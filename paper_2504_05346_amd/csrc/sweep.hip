// Column-block sweep of thanos_prune_layer: mask selection, per-row solve, trailing update.
//
// Per block [j1, j2) of B columns, with U the factor of thanos_factor (H_d^{-1} = U^T U):
//   P_k   = U[j1:j2, j1:j2]^T * U[j1:j2, j1:b]      first (j2-j1) rows of inv(H_d[j1:, j1:]),
//                                                   i.e. every row "R" of Sec. 4.1 can need
//   G     = P_k[:, 0:j2-j1]                          so that R_hat = G[q, q]
//   lambda R_hat = u, u = W[i, j1+q]                 per-row solve (eq. (R_hat), (u))
//   Lam[i, q] = lambda, 0 elsewhere                  scattered multipliers
//   W[:, j1:b] -= Lam * P_k                          == -u R_hat^{-1} R for every row at once
// All P_k are produced by one batched launch before the sweep.
#include <algorithm>

#include <cmath>

#include "gemm_tile_x3.h"

namespace thanos {

// Orders LDS traffic between the lanes of ONE wavefront (no instruction beyond a wait).
#define WAVE_SYNC()                                        \
  do {                                                     \
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); \
    __builtin_amdgcn_wave_barrier();                       \
  } while (0)

// The value of lane (l & 31) for every lane l: the lower half of the wavefront broadcast to the
// upper half (one v_permlane32_swap, no trip through LDS).
__device__ __forceinline__ float lower_half(float v) {
  const unsigned int u = __float_as_uint(v);
  return __uint_as_float(__builtin_amdgcn_permlane32_swap(u, u, false, false)[0]);
}

// ------------------------------------------------------------------------------------------
// small helpers
__global__ void k_fill_u32(uint32_t* p, int64_t n, uint32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

template <typename T>
__device__ __forceinline__ float load_as_float(const T* p);
template <>
__device__ __forceinline__ float load_as_float<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_as_float<__half>(const __half* p) { return __half2float(*p); }
template <>
__device__ __forceinline__ float load_as_float<__hip_bfloat16>(const __hip_bfloat16* p) {
  return __bfloat162float(*p);
}

template <typename T>
__global__ __launch_bounds__(256) void k_to_f32(const T* __restrict__ in, float* __restrict__ out,
                                                int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = load_as_float<T>(in + i);
}

template <typename T>
__global__ __launch_bounds__(256) void k_from_f32(const float* __restrict__ in, T* __restrict__ out,
                                                  int64_t n);
template <>
__global__ __launch_bounds__(256) void k_from_f32<__half>(const float* __restrict__ in,
                                                          __half* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = __float2half_rn(in[i]);
}
template <>
__global__ __launch_bounds__(256) void k_from_f32<__hip_bfloat16>(const float* __restrict__ in,
                                                                  __hip_bfloat16* __restrict__ out,
                                                                  int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = __float2bfloat16(in[i]);
}
template <>
__global__ __launch_bounds__(256) void k_from_f32<float>(const float* __restrict__ in,
                                                         float* __restrict__ out, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) out[i] = in[i];
}

__global__ __launch_bounds__(256) void k_sqrt(const float* __restrict__ xn2, float* __restrict__ sx,
                                              int64_t b) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j < b) sx[j] = sqrtf(xn2[j]);
}

// ------------------------------------------------------------------------------------------
// P[(j1+m)*b + col] = sum_k U[j1+k][j1+m] * U[j1+k][col], col in [j1, b), for every block.
struct BlockRowsArgs {
  const float* U;
  float* P;
  int64_t b;
  int B;
  int vec;
};

__global__ __launch_bounds__(kXThreads, 4) void k_block_rows(BlockRowsArgs a) {
  extern __shared__ __attribute__((aligned(16))) char sm[];
  const int64_t j1 = (int64_t)blockIdx.y * a.B;
  const int bw = (int)min((int64_t)a.B, a.b - j1);
  const int64_t col0 = j1 + (int64_t)blockIdx.x * kTN;
  const int mrow0 = (int)blockIdx.z * kTM;  // row tile inside the block (B may exceed 128)
  if (col0 >= a.b || mrow0 >= bw) return;
  const int n_ext = (int)min((int64_t)kTN, a.b - col0);
  const int m_ext = min(kTM, bw - mrow0);
  const float* A = a.U + j1 * a.b + j1 + mrow0;  // (m,k) at A[k*b + m]
  const float* Bm = a.U + j1 * a.b + col0;       // (k,n) at B[k*b + n]
  TileAcc acc;
  acc_zero(acc);
  gemm_tile_x3<true, true>(acc, sm, A, a.b, m_ext, Bm, a.b, n_ext, 0, bw, a.vec, a.vec);
  float* Pg = a.P + (j1 + mrow0) * a.b + col0;
  if (m_ext == kTM && n_ext == kTN && a.vec) {  // P is 256-byte aligned, b and col0 multiples of 4
    x3_write_tile(acc, sm, Pg, a.b, 1.f);
    return;
  }
  const float* T = x3_stage_tile(acc, sm);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int i = 0; i < 16; ++i) {
    const int row = wave + 8 * i;
    if (row >= m_ext) break;
#pragma unroll
    for (int e = 0; e < 2; ++e)
      if (2 * lane + e < n_ext) Pg[(int64_t)row * a.b + 2 * lane + e] = T[row * kXCLd + 2 * lane + e];
  }
}

// ------------------------------------------------------------------------------------------
// Inverses of the blocks' G matrices, for rows that lose more than half of a block.
// With G = P_k[:, :bw] = U_bb^T U_bb (U_bb the diagonal block of the factor), K = G^{-1} =
// V_bb V_bb^T, where V = U^{-1} is the reverse Cholesky factor the factorisation leaves behind
// (V[x][y] = L[b-1-x][b-1-y], L = its workspace's lower factor of the index-reversed matrix), and
// the diagonal block of the inverse of a triangular matrix is the inverse of its diagonal block:
// no inversion is computed.  Kc[blk][a][j] = sum_{m >= max(a, j)} V[j1+a][j1+m] V[j1+j][j1+m],
// row stride B.  One workgroup per 32 x 32 tile of a block.
__global__ __launch_bounds__(256) void k_comp_blocks(const float* __restrict__ L, int64_t ldL,
                                                     int64_t b, int B, float* __restrict__ Kc) {
  __shared__ float Va[32][33], Vj[32][33];
  const int64_t j1 = (int64_t)blockIdx.z * B;
  const int bw = (int)min((int64_t)B, b - j1);
  const int a0 = 32 * blockIdx.y, c0 = 32 * blockIdx.x;
  if (a0 >= bw || c0 >= bw) return;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // ty 0..7
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  auto V = [&](int x, int y) -> float {  // block-local indices, zero outside the upper triangle
    if (x >= bw || y >= bw || y < x) return 0.f;
    return L[(b - 1 - (j1 + x)) * ldL + (b - 1 - (j1 + y))];
  };
  for (int m0 = (max(a0, c0) / 32) * 32; m0 < bw; m0 += 32) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      Va[ty + 8 * e][tx] = V(a0 + ty + 8 * e, m0 + tx);
      Vj[ty + 8 * e][tx] = V(c0 + ty + 8 * e, m0 + tx);
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float t = acc[e];
#pragma unroll
      for (int m = 0; m < 32; ++m) t = fmaf(Va[ty + 8 * e][m], Vj[tx][m], t);
      acc[e] = t;
    }
    __syncthreads();
  }
  float* out = Kc + (int64_t)blockIdx.z * B * B;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (a0 + ty + 8 * e < bw && c0 + tx < bw) out[(int64_t)(a0 + ty + 8 * e) * B + c0 + tx] = acc[e];
}

// ------------------------------------------------------------------------------------------
// Unstructured selection: exact r-th smallest metric over the residual W[:, j1:b] by a radix
// select on the fp32 bit pattern (11 + 11 + 10 bits), all state on the device.
//
// ONE launch per block (k_select), at most one workgroup per compute unit so that all of them
// are resident at once.  The threshold of a block is predicted from the previous block's: the
// update that writes the new weights also histograms a window of 2048 bins (of 16 to 64 keys)
// around the previous tau, counts what lies below it, and every update workgroup lists the keys of its
// tile that fall inside the window (with their rows).  Every workgroup of k_select works out for
// itself, from the same data, whether the wanted rank falls inside the window.
//   * It does (every block after the first on all data tried): the bin gives all but the last
//     4 to 6 bits of tau.
//     The workgroups go through the per-tile lists in parallel and hand the keys of that bin to
//     workgroup 0, which resolves the last bits and the ties from them: no pass over the
//     weights, and no device-wide fence (on this chip a release fence at device scope writes the
//     L2 of a compute die back, ~20 us after an update has filled it; the hand-over uses atomic
//     stores, loads and counters only, which are coherent across the dies by themselves).
//   * It does not (first block, a threshold that moved out of the window, a full list): all
//     workgroups run the three radix passes over the residual, separated by grid-wide barriers.
// Every wait is bounded: a wait that does not end within kSpinMax polls ends the kernel and
// reports kInfoSelectTimeout through info, so no wave can spin for ever.  Waiting workgroups
// poll a word of their own (or, for the one counter workgroup 0 waits on, are alone in polling):
// hundreds of pollers on one address make every access to that cache line take microseconds.
// The counters of a launch (arrivals, barrier, bin list) are cleared by the update that runs
// between two launches, never by k_select itself, so no workgroup can meet a counter that
// another one has already reset.
struct SelState {
  long long r_rem;      // weights still to remove (before the current block)
  long long need_eq;    // how many keys equal to tau are removed (ties, in (row, col) order)
  int ties_all;         // every key equal to tau is removed: no ranking of ties (need_eq = 2^62)
  int deferred;         // 1: some row of the block was left to the second solver launch
  unsigned int tau;     // r-th smallest key
  int none;             // 1: nothing left to remove
  unsigned int win_lo;  // first bin (key >> win_shift) of the window of the NEXT block
  int win_shift;        // keys per bin of that window = 2^win_shift (kWinShiftMin .. kWinShiftMax)
  int pred_try;         // 1: a window was counted for this block
  int cand_overflow;    // an update workgroup found more window keys than it can list
  // counters of the current k_select launch
  unsigned int arrived; // workgroups that have handed over their part
  unsigned int nbin;    // keys of the threshold's bin handed to workgroup 0
  unsigned int bar;     // arrivals at the grid barriers
};

constexpr int32_t kInfoSelectTimeout = -0x7ffffff0;  // info: a bounded wait of k_select ran out
constexpr int kSelThreads = 1024;
constexpr int kSelMaxWgs = 256;       // at most one per compute unit: all resident at once
constexpr unsigned int kSpinMax = 1u << 21;
constexpr int kCandStage = 384;       // window keys one update workgroup can list (two update
                                      // workgroups still fit the LDS of a compute unit)
constexpr int kBinCap = 4096;         // keys of the threshold's bin that k_select can resolve
// The window has 2048 bins of 2^shift keys, 1024 on either side of the last threshold.  The bin
// width follows the drift of the threshold from block to block (at least 8 times the last step
// must fit into half the window): 16 keys per bin (+- 0.2 % of tau) while the threshold moves
// little, up to 64 (+- 0.8 %) when it moves more; the lists of window keys grow in proportion,
// which is what bounds the width.
constexpr int kWinShiftMin = 4, kWinShiftMax = 6;

__device__ __forceinline__ unsigned int metric_key(float w, float sx) {
  return __float_as_uint(fabsf(w) * sx);
}

// Workgroup of NT threads: the bin of hist[0 .. nbins) (nbins = 16, 1024 or 2048) that holds
// the rank-th smallest key, the number of keys in the bins before it and inside it.  bin = -1
// if rank is not in 1 .. total.
struct BinSel {
  int bin;
  unsigned int count;
  long long before;
};
template <int NT>
__device__ __forceinline__ BinSel block_select_bin(const unsigned int* __restrict__ hist,
                                                   int nbins, long long rank) {
  __shared__ long long wtot[NT / 64];
  __shared__ BinSel res;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = nbins >= NT ? nbins / NT : 1;  // at most 8
  unsigned int loc[8];
  long long s = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int idx = tid * per + e;
    loc[e] = (e < per && idx < nbins) ? hist[idx] : 0u;
    s += loc[e];
  }
  long long incl = s;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long t = __shfl_up(incl, off, 64);
    if (lane >= off) incl += t;
  }
  if (lane == 63) wtot[wave] = incl;
  if (tid == 0) res.bin = -1;
  __syncthreads();
  long long before = incl - s;
  for (int v = 0; v < wave; ++v) before += wtot[v];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (rank > 0 && before < rank && rank <= before + loc[e]) {
      res.bin = tid * per + e;
      res.count = loc[e];
      res.before = before;
    }
    before += loc[e];
  }
  __syncthreads();
  const BinSel r = res;
  __syncthreads();  // res and wtot are free for the next call
  return r;
}

// Sum of one value per thread over a workgroup of NT threads (all threads get it).
template <int NT>
__device__ __forceinline__ long long block_sum(long long v) {
  __shared__ long long wsum[NT / 64];
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
  __syncthreads();
  long long t = 0;
  for (int w = 0; w < NT / 64; ++w) t += wsum[w];
  __syncthreads();
  return t;
}

// PASS 0: bin = key >> 21.  PASS 1: keys with key>>21 == prefix, bin = (key>>10) & 2047.
// PASS 2: keys with key>>10 == prefix, bin = the low 10 bits; also counts those keys (cand).
template <int PASS>
__device__ __forceinline__ void sel_count(unsigned int* h, unsigned int key, unsigned int prefix,
                                          int& cand) {
  if (PASS == 0) {
    atomicAdd(&h[key >> 21], 1u);
  } else if (PASS == 1) {
    if ((key >> 21) == prefix) atomicAdd(&h[(key >> 10) & 2047u], 1u);
  } else {
    if ((key >> 10) == prefix) {
      atomicAdd(&h[key & 1023u], 1u);
      ++cand;
    }
  }
}

struct SelectArgs {
  const float* W;
  const float* sx;
  SelState* st;
  unsigned int* hist;              // window histogram, then the three radix passes (4 x 2048)
  const unsigned int* below_part;  // keys below the window, one count per update workgroup
  int n_part;                      // update workgroups (tiles) of the previous block
  const unsigned int* cand_n;      // per tile: keys inside the window
  const uint2* cand;               // per tile: kCandStage x (key, row)
  unsigned long long* binlist;     // kBinCap x (row << 32 | key): the threshold's bin
  const int* row_cnt;              // weights the previous block removed from each row
  int* row_cand;                   // per row: keys sharing the bits resolved before the last pass
  int* row_eq;                     // per row: keys equal to tau, then their exclusive prefix
  float* tau_out;                  // optional: threshold of this block
  int32_t* info;
  int64_t c, b, j1;
  int first;                       // first block: no window exists
  int vec;                         // 16-byte loads of the row segments are aligned
  unsigned int seq;                // block sequence number, >= 1
  // One word per workgroup, each in a cache line of its own (stride kFlagStride), through which
  // a grid barrier releases it.  Values only grow: 8 * seq + k after barrier k of block seq.
  unsigned int* wgflag;
};
constexpr int kFlagStride = 32;  // words (128 bytes)

// Thread 0 of the calling workgroup waits until *f has reached `want` (bounded).
__device__ __forceinline__ unsigned int wait_word(const unsigned int* f, unsigned int want) {
  unsigned int n = 0, v = 0;
  for (;;) {
    v = __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (v >= want || ++n >= kSpinMax) break;
    __builtin_amdgcn_s_sleep(8);
  }
  return v;
}

// One radix pass of the calling workgroup over its rows (one wavefront per row; lanes stride
// over the residual columns, 16 bytes per lane when aligned).  The workgroup's LDS histogram h
// is added to hist_out at the end.
template <int PASS>
__device__ __forceinline__ void sel_pass(const SelectArgs& a, unsigned int* h, unsigned int prefix,
                                         unsigned int* __restrict__ hist_out) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int e = tid; e < 2048; e += kSelThreads) h[e] = 0u;
  __syncthreads();
  constexpr int RW = kSelThreads / 64;  // rows per workgroup and step
  for (int64_t i = (int64_t)blockIdx.x * RW + wave; i < a.c; i += (int64_t)gridDim.x * RW) {
    const float* row = a.W + i * a.b;
    int cand = 0;
    if (a.vec) {
      const int64_t nvec = (a.b - a.j1) >> 2;
      for (int64_t v = lane; v < nvec; v += 64) {
        const int64_t j = a.j1 + 4 * v;
        const float4 w4 = *reinterpret_cast<const float4*>(row + j);
        const float4 s4 = *reinterpret_cast<const float4*>(a.sx + j);
        sel_count<PASS>(h, metric_key(w4.x, s4.x), prefix, cand);
        sel_count<PASS>(h, metric_key(w4.y, s4.y), prefix, cand);
        sel_count<PASS>(h, metric_key(w4.z, s4.z), prefix, cand);
        sel_count<PASS>(h, metric_key(w4.w, s4.w), prefix, cand);
      }
      for (int64_t j = a.j1 + 4 * nvec + lane; j < a.b; j += 64)
        sel_count<PASS>(h, metric_key(row[j], a.sx[j]), prefix, cand);
    } else {
      for (int64_t j = a.j1 + lane; j < a.b; j += 64)
        sel_count<PASS>(h, metric_key(row[j], a.sx[j]), prefix, cand);
    }
    if (PASS == 2) {
      for (int off = 32; off > 0; off >>= 1) cand += __shfl_down(cand, off, 64);
      if (lane == 0) a.row_cand[i] = cand;
    }
  }
  __syncthreads();
  for (int e = tid; e < 2048; e += kSelThreads)
    if (h[e]) atomicAdd(&hist_out[e], h[e]);
}

// All workgroups of the launch have arrived at barrier `phase` (1, 2, ...) of this block: each
// adds itself to a counter, and the one that completes the count releases every workgroup
// through its own word.  Release and acquire fences at device scope on both sides: what the
// workgroups wrote before the barrier (histogram atomics, per-row counts) is read after it.
// Returns false if the wait ran out.
__device__ __forceinline__ bool grid_barrier(const SelectArgs& a, unsigned int phase) {
  __shared__ int ok, last;
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence();
    last = atomicAdd(&a.st->bar, 1u) + 1u == phase * gridDim.x ? 1 : 0;
  }
  __syncthreads();
  const unsigned int want = 8u * a.seq + phase;
  if (last)
    for (unsigned int w = threadIdx.x; w < gridDim.x; w += kSelThreads)
      __hip_atomic_store(a.wgflag + (size_t)w * kFlagStride, want, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
  if (threadIdx.x == 0)
    ok = wait_word(a.wgflag + (size_t)blockIdx.x * kFlagStride, want) >= want ? 1 : 0;
  __syncthreads();
  __threadfence();
  return ok != 0;
}

// Exclusive prefix sum of row_eq over the rows by one workgroup, in place: afterwards row_eq[i]
// = number of keys equal to tau in the rows before row i (ties are taken in (row, column) order).
__device__ __forceinline__ void tie_prefix(int* __restrict__ row_eq, int64_t c) {
  __shared__ long long wtot[kSelThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t per = (c + kSelThreads - 1) / kSelThreads;
  const int64_t lo = tid * per, hi = min(c, lo + per);
  long long s = 0;
  for (int64_t i = lo; i < hi; ++i) s += row_eq[i];
  long long incl = s;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long t = __shfl_up(incl, off, 64);
    if (lane >= off) incl += t;
  }
  if (lane == 63) wtot[wave] = incl;
  __syncthreads();
  long long run = incl - s;
  for (int v = 0; v < wave; ++v) run += wtot[v];
  for (int64_t i = lo; i < hi; ++i) {
    const int v = row_eq[i];
    row_eq[i] = (int)min(run, (long long)0x7fffffff);
    run += v;
  }
}

// Workgroup 0, at the end of the launch: the state later kernels read.  tau_valid: a threshold
// was found (else nothing is left to remove).
__device__ __forceinline__ void publish(const SelectArgs& a, long long r_rem, bool tau_valid,
                                        unsigned int tau, long long rank_eq, bool all) {
  SelState* st = a.st;
  for (int e = threadIdx.x; e < 2048; e += kSelThreads) a.hist[e] = 0u;  // window: consumed
  if (threadIdx.x != 0) return;
  st->r_rem = r_rem;
  st->none = tau_valid ? 0 : 1;
  st->deferred = 0;
  st->cand_overflow = 0;
  if (!tau_valid) {
    if (a.tau_out) *a.tau_out = -1.f;
    return;
  }
  // bin width of the next window from the step the threshold has just taken
  int shift = kWinShiftMin;
  if (!a.first && st->tau != 0u) {
    const unsigned int prev = st->tau;
    const unsigned int step = tau > prev ? tau - prev : prev - tau;
    while (shift < kWinShiftMax && (1024u << shift) < 8u * (unsigned long long)step) ++shift;
  }
  st->tau = tau;
  if (a.tau_out) *a.tau_out = __uint_as_float(tau);
  st->need_eq = all ? (1ll << 62) : rank_eq;
  st->ties_all = all ? 1 : 0;
  const unsigned int pb = tau >> shift;
  st->pred_try = tau != 0u ? 1 : 0;
  st->win_shift = shift;
  st->win_lo = pb > 1024u ? pb - 1024u : 0u;
}

__global__ __launch_bounds__(kSelThreads) void k_select(SelectArgs a) {
  __shared__ unsigned int h[2048];
  __shared__ unsigned long long bins[kBinCap];  // workgroup 0: the threshold's bin
  __shared__ unsigned int h16[1 << kWinShiftMax];  // counts of the bin's keys by their low bits
  __shared__ unsigned int s_ok;
  SelState* st = a.st;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  constexpr int RW = kSelThreads / 64;

  // ---- every workgroup: r <- r - ||M||_F^2 of the previous block (Alg. 1), the keys below the
  //      window, and whether the window holds the wanted rank.  Nothing read here is written
  //      before all workgroups have handed over (workgroup 0 writes the state at the very end).
  long long sum = 0, bsum = 0;
  if (!a.first) {
    for (int64_t i = tid; i < a.c; i += kSelThreads) sum += a.row_cnt[i];
    for (int e = tid; e < a.n_part; e += kSelThreads) bsum += a.below_part[e];
  }
  const long long r_old = st->r_rem;
  const bool pred_try = !a.first && st->pred_try != 0 && st->cand_overflow == 0;
  const unsigned int win_lo = st->win_lo;
  const int wsh = st->win_shift;
  const long long r_rem = r_old - block_sum<kSelThreads>(sum);
  const long long below = block_sum<kSelThreads>(bsum);
  const bool none = r_rem <= 0;
  BinSel r;
  r.bin = -1;
  r.count = 0;
  r.before = 0;
  if (!none && pred_try) r = block_select_bin<kSelThreads>(a.hist, 2048, r_rem - below);
  const bool hit = r.bin >= 0 && r.count <= (unsigned int)kBinCap;

  if (none || hit) {
    if (hit) {
      // ---- the keys of the threshold's bin: one wavefront per tile list; the list of a tile
      //      holds at most kCandStage entries, i.e. up to 6 independent loads per lane ----
      const unsigned int prefix28 = win_lo + (unsigned int)r.bin;
      for (int t = (int)blockIdx.x * RW + wave; t < a.n_part; t += (int)gridDim.x * RW) {
        const unsigned int n = min(a.cand_n[t], (unsigned int)kCandStage);
        const uint2* list = a.cand + (size_t)t * kCandStage;
        uint2 kr[kCandStage / 64];
#pragma unroll
        for (int u = 0; u < kCandStage / 64; ++u) kr[u] = list[min(64 * u + lane, kCandStage - 1)];
#pragma unroll
        for (int u = 0; u < kCandStage / 64; ++u)
          if ((unsigned int)(64 * u + lane) < n && (kr[u].x >> wsh) == prefix28) {
            const unsigned int slot = atomicAdd(&st->nbin, 1u);
            if (slot < (unsigned int)kBinCap)
              __hip_atomic_store(a.binlist + slot,
                                 ((unsigned long long)kr[u].y << 32) | kr[u].x, __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
          }
      }
    }
    // hand over: this workgroup's entries have left before it counts itself in
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    if (tid == 0) atomicAdd(&st->arrived, 1u);
    if (blockIdx.x != 0) return;

    // ---- workgroup 0: wait for the others (it is the only one polling this counter) ----
    if (tid == 0) s_ok = wait_word(&st->arrived, gridDim.x) >= gridDim.x ? 1u : 0u;
    __syncthreads();
    if (!s_ok) {
      if (tid == 0) atomicCAS(a.info, 0, kInfoSelectTimeout);
      return;
    }
    if (none) {
      publish(a, r_rem, false, 0u, 0, true);
      return;
    }
    const unsigned int nbin = __hip_atomic_load(&st->nbin, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (nbin != r.count) {  // the lists and the histogram disagree: cannot happen
      if (tid == 0) atomicCAS(a.info, 0, kInfoSelectTimeout);
      return;
    }
    const unsigned int nlow = 1u << wsh;
    if (tid < (int)nlow) h16[tid] = 0u;
    __syncthreads();
    for (unsigned int e = tid; e < nbin; e += kSelThreads) {
      const unsigned long long v =
          __hip_atomic_load(a.binlist + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      bins[e] = v;
      atomicAdd(&h16[(unsigned int)v & (nlow - 1u)], 1u);
    }
    __syncthreads();
    long long rank = r_rem - below - r.before;  // 1-based rank inside the bin
    unsigned int low = 0, cnt_eq = 0;
    for (unsigned int v = 0; v < nlow; ++v) {   // uniform: every thread walks the counts
      if (rank <= (long long)h16[v]) {
        low = v;
        cnt_eq = h16[v];
        break;
      }
      rank -= h16[v];
    }
    const unsigned int prefix28 = win_lo + (unsigned int)r.bin;
    const unsigned int tau = (prefix28 << wsh) | low;
    const bool all = rank == (long long)cnt_eq;
    if (!all) {
      // ties to rank (some, not all, keys equal to tau are removed), in (row, column) order:
      // row_eq[i] = keys equal to tau in the rows before row i, counted from the bin in LDS
      for (int64_t i = tid; i < a.c; i += kSelThreads) {
        int before = 0;
        for (unsigned int e = 0; e < nbin; ++e)
          before += ((unsigned int)bins[e] == tau && (unsigned int)(bins[e] >> 32) < (unsigned int)i) ? 1 : 0;
        a.row_eq[i] = before;
      }
    }
    publish(a, r_rem, true, tau, rank, all);
    return;
  }

  // ---- radix passes over the residual, all workgroups (the histograms of the passes were
  //      cleared by the update, or by the fill at the start of the sweep) ----
  unsigned int* hist_a = a.hist + 2048;
  unsigned int* hist_b = a.hist + 2 * 2048;
  unsigned int* hist_c = a.hist + 3 * 2048;
  bool ok = true;
  sel_pass<0>(a, h, 0u, hist_a);
  ok = grid_barrier(a, 1u);
  const BinSel r0 = block_select_bin<kSelThreads>(hist_a, 2048, r_rem);
  const unsigned int prefix1 = (unsigned int)r0.bin;
  const long long rank1 = r_rem - r0.before;
  if (ok) {
    sel_pass<1>(a, h, prefix1, hist_b);
    ok = grid_barrier(a, 2u);
  }
  const BinSel r1 = block_select_bin<kSelThreads>(hist_b, 2048, rank1);
  const unsigned int prefix2 = (prefix1 << 11) | (unsigned int)r1.bin;
  const long long rank2 = rank1 - r1.before;
  if (ok) {
    sel_pass<2>(a, h, prefix2, hist_c);
    ok = grid_barrier(a, 3u);
  }
  if (!ok) {
    if (tid == 0) atomicCAS(a.info, 0, kInfoSelectTimeout);
    return;
  }
  // The last pass resolves the key completely, so the chosen bin counts the keys equal to tau:
  // if all of them are removed (the usual case: one key at the threshold) their order does not
  // matter and nothing is ranked.
  const BinSel r2 = block_select_bin<kSelThreads>(hist_c, 1024, rank2);
  const unsigned int tau = (prefix2 << 10) | (unsigned int)r2.bin;
  const long long rank_eq = rank2 - r2.before;  // keys equal to tau that are removed
  const bool all = rank_eq == (long long)r2.count;
  if (all) {
    if (blockIdx.x == 0) publish(a, r_rem, true, tau, rank_eq, true);
    return;
  }
  // rows that hold candidates (keys sharing the 22 bits resolved before the last pass) count
  // their keys equal to tau over the residual row; other rows have none
  for (int64_t i = (int64_t)blockIdx.x * RW + wave; i < a.c; i += (int64_t)gridDim.x * RW) {
    int n = 0;
    if (a.row_cand[i] != 0) {
      const float* row = a.W + i * a.b;
      if (a.vec) {
        const int64_t nvec = (a.b - a.j1) >> 2;
        for (int64_t v = lane; v < nvec; v += 64) {
          const int64_t j = a.j1 + 4 * v;
          const float4 w4 = *reinterpret_cast<const float4*>(row + j);
          const float4 s4 = *reinterpret_cast<const float4*>(a.sx + j);
          n += (metric_key(w4.x, s4.x) == tau) + (metric_key(w4.y, s4.y) == tau) +
               (metric_key(w4.z, s4.z) == tau) + (metric_key(w4.w, s4.w) == tau);
        }
        for (int64_t j = a.j1 + 4 * nvec + lane; j < a.b; j += 64)
          n += (metric_key(row[j], a.sx[j]) == tau) ? 1 : 0;
      } else {
        for (int64_t j = a.j1 + lane; j < a.b; j += 64)
          n += (metric_key(row[j], a.sx[j]) == tau) ? 1 : 0;
      }
      for (int off = 32; off > 0; off >>= 1) n += __shfl_down(n, off, 64);
    }
    if (lane == 0) a.row_eq[i] = n;
  }
  if (!grid_barrier(a, 4u)) {
    if (tid == 0) atomicCAS(a.info, 0, kInfoSelectTimeout);
    return;
  }
  if (blockIdx.x == 0) {
    tie_prefix(a.row_eq, a.c);
    publish(a, r_rem, true, tau, rank_eq, false);
  }
}

// Ties before row i; row_eq is stale (and not read) when no tie needs ranking.
__device__ __forceinline__ long long ties_before(const SelState* __restrict__ st,
                                                 const int* __restrict__ row_eq, int64_t i) {
  return (st->none || st->ties_all) ? 0 : (long long)row_eq[i];
}

// ------------------------------------------------------------------------------------------
// Mask + per-row solve (Alg. 1, loop over the rows of W; Sec. 4.1, eqs. (R_hat), (u)):
// lambda R_hat = u with R_hat = G[q, q], G the block's rows of the residual inverse, q the
// removed columns of the row (Sec. 4.5), u the removed weights.  Three kernels share the
// arguments below and differ in how many unknowns they hold and where.
enum { SEL_NM = 0, SEL_THRESHOLD = 1, SEL_GIVEN = 2 };

struct SolveArgs {
  const float* W;        // c x b, current weights
  const float* P;        // b x b, block rows of the residual inverses
  const float* sx;       // sqrt(xnorm2)
  const uint8_t* mask_in;
  uint8_t* mask_out;     // c x b
  float* Lam;            // c x ldl
  const SelState* st;    // SEL_THRESHOLD
  SelState* st_rw;
  const int* row_eq;     // exclusive tie prefix per row (k_select; see ties_before)
  int* row_cnt;          // SEL_THRESHOLD: number of weights removed from row i in this block
  const uint8_t* row_skip;  // optional, c bytes: 1 = row is left untouched (outlier row)
  int32_t* info;
  int64_t c, b, j1;
  int bw, ldl, n, m;
  int nt_lo, nt_max;     // k_solve_tiled: rows with nt_lo <= ceil(s/32) <= nt_max; LDS holds nt_max
  int s_min;             // k_solve_wide: rows with s < s_min belong to another launch
  float* tile_scratch;   // k_solve_tiled<.., BIG>: tile grids in global memory, one slot per workgroup
  int64_t slot_floats;
  const float* Kc;       // k_solve_tiled: inverse of this block's G (bw x bw, row stride ldk), or
  int ldk;               // nullptr; rows that lose more than half of the block are solved through it
  int defer_large;       // k_solve_mfma: rows with more unknowns than it holds belong to another launch
};

// ------------------------------------------------------------------------------------------
// Mask + per-row solve for systems of up to SMAX = 128 or 256 unknowns: one workgroup of SMAX
// threads (2 or 4 wavefronts) per row of W, thread t <-> block column t <-> row t of R_hat
// (SMAX registers).
// Symmetric Gauss-Jordan elimination (no back-substitution: after s steps lambda_k = u_k / d_k)
// in its square-root-free form  A[rho][j] -= (A[rho][k] / d) * A[j][k],  so that the broadcast
// column needs no scaling; after every panel of 4 pivots the registers are renamed (column j
// moves to register j - 4), which keeps all register indices static.  The pivot column travels
// through LDS (one barrier per pivot).
// Only the registers that still hold live columns (j < s - 4*panel) are touched, in chunks of
// 16, so a system of s unknowns costs ~s^2/2 fused multiply-adds per thread, not s*128.
template <int SEL, int SMAX>
__global__ __launch_bounds__(SMAX, (SMAX == 128 ? 3 : 1)) void k_solve_wide(SolveArgs a) {
  constexpr int NWV = SMAX / 64;
  __shared__ __attribute__((aligned(16))) float col[2][4][SMAX + 32];  // tail stays zero
  __shared__ float ukb[2][4];
  __shared__ float wrow[SMAX];
  __shared__ float key[SMAX];
  __shared__ int q[SMAX];
  __shared__ int cnt[NWV];
  __shared__ int eqc[NWV];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t i = blockIdx.x;
  const float* wrow_g = a.W + i * a.b + a.j1;
  // second launch of a block (s_min > 0): nothing to do unless the first one left rows behind
  if (SEL == SEL_THRESHOLD && a.s_min > 0 && a.st->deferred == 0) return;

  const float w = (tid < a.bw) ? wrow_g[tid] : 0.f;
  wrow[tid] = w;
  for (int e = tid; e < 2 * 4 * (SMAX + 32); e += SMAX) (&col[0][0][0])[e] = 0.f;
  bool sel = false;
  if (SEL == SEL_GIVEN) {
    sel = (tid < a.bw) && a.mask_in[i * a.b + a.j1 + tid] != 0;
  } else if (SEL == SEL_NM) {
    key[tid] = (tid < a.bw) ? fabsf(w) * a.sx[a.j1 + tid] : 0.f;
    __syncthreads();
    if (tid < a.bw) {
      const int g0 = (tid / a.m) * a.m;
      const float mine = key[tid];
      int rank = 0;
      for (int e = 0; e < a.m; ++e) {
        const float o = key[g0 + e];
        rank += (o < mine || (o == mine && g0 + e < tid)) ? 1 : 0;
      }
      sel = rank < a.n;
    }
    if (a.row_skip && a.row_skip[i]) sel = false;
  } else {  // SEL_THRESHOLD
    const bool none = a.st->none != 0;
    const unsigned int tau = a.st->tau;
    const long long need_eq = a.st->need_eq;
    const bool in = (tid < a.bw) && !none;
    const unsigned int kk = in ? metric_key(w, a.sx[a.j1 + tid]) : 0xffffffffu;
    const bool lt = in && kk < tau;
    const bool eq = in && kk == tau;
    const unsigned long long eqb = __ballot(eq);
    if (lane == 0) eqc[wave] = __popcll(eqb);
    __syncthreads();
    int eq_before = 0;
    for (int v = 0; v < wave; ++v) eq_before += eqc[v];
    const long long my = ties_before(a.st, a.row_eq, i) + eq_before +
                         __popcll(eqb & ((1ull << lane) - 1ull));
    sel = lt || (eq && my < need_eq);
  }
  const unsigned long long bal = __ballot(sel);
  if (lane == 0) cnt[wave] = __popcll(bal);
  __syncthreads();
  int s = 0, sel_before = 0;
  for (int v = 0; v < NWV; ++v) {
    if (v < wave) sel_before += cnt[v];
    s += cnt[v];
  }
  if (s < a.s_min) return;  // solved by the launch for smaller systems
  const int myrank = sel_before + __popcll(bal & ((1ull << lane) - 1ull));
  if (sel) q[myrank] = tid;
  if (tid < a.bw) a.mask_out[i * a.b + a.j1 + tid] = sel ? 1 : 0;
  if (SEL == SEL_THRESHOLD) {
    if (tid == 0) a.row_cnt[i] = s;  // summed at the start of the next block
  }
  float* lam_g = a.Lam + i * a.ldl;
  if (s == 0) {
    if (tid < a.bw) lam_g[tid] = 0.f;
    return;
  }
  __syncthreads();

  // ---- gather R_hat: A[j] = G[q_j][q_rho] (= G[q_rho][q_j]) ----
  const float* G = a.P + a.j1 * a.b + a.j1;
  const int rho = tid;
  const int qr = (rho < s) ? q[rho] : 0;
  float u = (rho < s) ? wrow[qr] : 0.f;
  float dinv = 0.f;
  float A[SMAX];
  // Loads are issued unconditionally, 16 at a time, from clamped (valid) indices and masked
  // afterwards: a conditional load, or a select right behind a load, makes the compiler wait for
  // every outstanding load, i.e. one memory round trip per element.  q * b < 2^31.
  {
    const unsigned int bb = (unsigned int)a.b, qc = (unsigned int)qr;
#pragma unroll
    for (int c16 = 0; c16 < SMAX / 16; ++c16) {
      if (16 * c16 < s) {
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
          const int j = 16 * c16 + jj;
          A[j] = G[(unsigned int)q[min(j, s - 1)] * bb + qc];
        }
      } else {
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) A[16 * c16 + jj] = 0.f;
      }
    }
#pragma unroll
    for (int j = 0; j < SMAX; ++j) A[j] = (j < s && rho < s) ? A[j] : 0.f;
  }

  // ---- elimination ----
  bool bad = false;
  const int npanel = (s + 3) >> 2;
  for (int pnl = 0; pnl < npanel; ++pnl) {
    const int k0 = 4 * pnl;
    const int wact = s - k0;  // live registers: columns k0 .. s-1
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int k = k0 + t;
      float* cb = col[pnl & 1][t];
      cb[rho] = A[t];
      if (rho == k) ukb[pnl & 1][t] = u;
      __syncthreads();
      const float d = cb[k];
      const float uk = ukb[pnl & 1][t];
      float rd = 0.f;
      if (k < s) {
        if (d > 0.f) rd = 1.f / d;
        else bad = true;
      }
      float m = A[t] * rd;
      if (rho == k) {
        dinv = rd;
        m = 0.f;  // the pivot row itself is not modified
      }
      u = fmaf(-m, uk, u);
      const f32x4* cv = reinterpret_cast<const f32x4*>(&cb[k0]);  // register j <-> column k0 + j
      if (t < 3) {
#pragma unroll
        for (int c16 = 0; c16 < SMAX / 16; ++c16) {
          if (16 * c16 < wact) {
#pragma unroll
            for (int j4 = 4 * c16; j4 < 4 * c16 + 4; ++j4) {
              const f32x4 lb = cv[j4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const int j = 4 * j4 + e;
                if (j > t) A[j] = fmaf(-m, lb[e], A[j]);
              }
            }
          }
        }
      } else {
#pragma unroll
        for (int c16 = 0; c16 < SMAX / 16; ++c16) {
          if (16 * c16 < wact + 4) {
#pragma unroll
            for (int j4 = 4 * c16; j4 < 4 * c16 + 4; ++j4) {
              if (j4 >= 1) {
                const f32x4 lb = cv[j4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  const int j = 4 * j4 + e;
                  A[j - 4] = fmaf(-m, lb[e], A[j]);
                }
              }
            }
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) A[SMAX - 4 + e] = 0.f;
      }
    }
  }
  if (bad && tid == 0) atomicCAS(a.info, 0, -(int32_t)min(i + 1, (int64_t)0x7fffffff));

  // ---- lambda row: zeros except lambda_k = u_k / d_k at column q_k ----
  __syncthreads();
  wrow[tid] = 0.f;
  __syncthreads();
  if (rho < s) wrow[qr] = u * dinv;
  __syncthreads();
  if (tid < a.bw) lam_g[tid] = wrow[tid];
}

// ------------------------------------------------------------------------------------------
// Mask + per-row solve on the matrix cores for systems of up to 32 NTR unknowns (NTR = 2 or 3,
// block width <= 128): one wavefront per row of W.  R_hat is held in the accumulator layout of
// v_mfma_f32_32x32x2_f32 as the lower triangle of a grid of 32x32 tiles (identity on the unused
// part): diagonal tiles as they are, tile (i, j), i > j, transposed (register r of lane (lo, hi)
// = R_hat[32 i + lo][32 j + row(r, hi)]), so that column k of a tile below the pivot tile is
// again row k of the register tile.  Symmetric elimination, square-root free (R_hat = L~ D L~^T):
// row k of a symmetric tile in that layout is at once both operands of its rank-1 update, and
// rows k and k + 4 share a register (lower / upper half of the wavefront), so a PAIR of pivots
// of tile row p costs one MFMA per live tile (i, j), p <= j <= i; the cross-lane traffic is the
// broadcast of the pivots and one cross-lane read per tile row (the second pivot's row must
// first see the elimination of the first).  The right-hand side u is carried along (forward
// substitution: one FMA per tile row and pair), the columns of L~ go to LDS, and
// L~^T lambda = D^-1 y is solved afterwards by column sweeps that read one LDS row per unknown.
// NTR = 2 serves n:m at B = 128 (s = 64 for 2:4 and 4:8); NTR = 3 the unstructured mode at
// B = 128, where s scatters around 64.
template <int NTR>
struct SolveMfmaSmem {
  static constexpr int N = 32 * NTR;
  float L[N * (N - 1) / 2 + 64];  // strict lower triangle of L~, packed by rows
  float wrow[128];
  float key[128];
  unsigned char q[128];
  float dummy[128];
};

// FULL: the host knows that every row has either no unknown or exactly 32 NTR (n:m on a whole
// block): the padding logic folds away.
template <int SEL, int WPB, int NTR, bool FULL = false>
__global__ __launch_bounds__(64 * WPB, 2) void k_solve_mfma(SolveArgs a) {
  constexpr int CPL = 2;  // block width <= 128
  constexpr int NZ = (NTR + 1) / 2;  // registers holding y / d: rows 64 z + lane
  extern __shared__ __attribute__((aligned(16))) char solve_smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  SolveMfmaSmem<NTR>& sm = reinterpret_cast<SolveMfmaSmem<NTR>*>(solve_smem)[wave];
  const int lo = lane & 31, hi = lane >> 5;
  const int64_t i = (int64_t)blockIdx.x * WPB + wave;
  if (i >= a.c) return;
  const float* wrow_g = a.W + i * a.b + a.j1;

  // ---- selection of the block mask row M_i ----
  bool sel[CPL];
  float wv[CPL];
#pragma unroll
  for (int r = 0; r < CPL; ++r) {
    const int col = lane + 64 * r;
    wv[r] = (col < a.bw) ? wrow_g[col] : 0.f;
    sm.wrow[col] = wv[r];
    sel[r] = false;
  }
  if (SEL == SEL_GIVEN) {
#pragma unroll
    for (int r = 0; r < CPL; ++r) {
      const int col = lane + 64 * r;
      sel[r] = (col < a.bw) && a.mask_in[i * a.b + a.j1 + col] != 0;
    }
  } else if (SEL == SEL_NM) {
#pragma unroll
    for (int r = 0; r < CPL; ++r) {
      const int col = lane + 64 * r;
      sm.key[col] = (col < a.bw) ? fabsf(wv[r]) * a.sx[a.j1 + col] : 0.f;
    }
    WAVE_SYNC();
#pragma unroll
    for (int r = 0; r < CPL; ++r) {
      const int col = lane + 64 * r;
      if (col < a.bw) {
        const int g0 = (col / a.m) * a.m;
        const float mine = sm.key[col];
        int rank = 0;
        for (int e = 0; e < a.m; ++e) {
          const float o = sm.key[g0 + e];
          rank += (o < mine || (o == mine && g0 + e < col)) ? 1 : 0;
        }
        sel[r] = rank < a.n;
      }
    }
    if (a.row_skip && a.row_skip[i]) {
#pragma unroll
      for (int r = 0; r < CPL; ++r) sel[r] = false;
    }
  } else {  // SEL_THRESHOLD: key < tau, or key == tau and among the first need_eq ties
    const bool none = a.st->none != 0;
    const unsigned int tau = a.st->tau;
    const long long need_eq = a.st->need_eq;
    long long tie_rank = ties_before(a.st, a.row_eq, i);
#pragma unroll
    for (int r = 0; r < CPL; ++r) {
      const int col = lane + 64 * r;
      const bool in = (col < a.bw) && !none;
      const unsigned int key = in ? metric_key(wv[r], a.sx[a.j1 + col]) : 0xffffffffu;
      const bool lt = in && key < tau;
      const bool eq = in && key == tau;
      const unsigned long long eqb = __ballot(eq);
      const long long my = tie_rank + __popcll(eqb & ((1ull << lane) - 1ull));
      sel[r] = lt || (eq && my < need_eq);
      tie_rank += __popcll(eqb);
    }
  }

  // ---- q = phi(M_i) (ascending column indices) and s ----
  int s = 0;
  int myrank[CPL];
#pragma unroll
  for (int r = 0; r < CPL; ++r) {
    const unsigned long long bal = __ballot(sel[r]);
    myrank[r] = s + __popcll(bal & ((1ull << lane) - 1ull));
    s += __popcll(bal);
  }
  // A row with more unknowns than the tile grid holds (s > 32 NTR; rare): with the inverse K of
  // the block's G at hand it is solved here through the complement, a system of bw - s < 32
  // unknowns (see k_solve_tiled for the identity); without K it is left to the launch for
  // larger systems.
  bool comp = false;
  if (s > 32 * NTR && a.defer_large) {
    if (FULL || a.Kc == nullptr) {
      if (SEL == SEL_THRESHOLD && lane == 0) a.st_rw->deferred = 1;
      return;
    }
    comp = true;
  }
  const int ns = comp ? a.bw - s : s;  // unknowns of the system solved below
  if (comp) {  // positions of the KEPT columns of the block
    int before = 0;
#pragma unroll
    for (int r = 0; r < CPL; ++r) {
      const int col = lane + 64 * r;
      const bool kept = col < a.bw && !sel[r];
      const unsigned long long bal = __ballot(kept);
      if (kept) sm.q[before + __popcll(bal & ((1ull << lane) - 1ull))] = (unsigned char)col;
      before += __popcll(bal);
    }
  }
#pragma unroll
  for (int r = 0; r < CPL; ++r) {
    const int col = lane + 64 * r;
    if (sel[r] && !comp) sm.q[myrank[r]] = (unsigned char)col;
    if (col < a.bw) a.mask_out[i * a.b + a.j1 + col] = sel[r] ? 1 : 0;
  }
  if (SEL == SEL_THRESHOLD) {
    if (lane == 0) a.row_cnt[i] = s;  // summed at the start of the next block
  }
  float* lam_g = a.Lam + i * a.ldl;
  // s > 32 NTR (or, if FULL, anything but 32 NTR) cannot happen for a launch chosen by the host
  if (s == 0 || (s > 32 * NTR && !comp) || (FULL && s != 32 * NTR)) {
#pragma unroll
    for (int r = 0; r < CPL; ++r) {
      const int col = lane + 64 * r;
      if (col < a.bw) lam_g[col] = 0.f;
    }
    return;
  }
  // y[r] = sum_a x[a] K[a][lane + 64 r] for this wavefront (x in LDS, zeros skipped)
  auto matvec_k = [&](const float* x, float (&y)[CPL]) {
#pragma unroll
    for (int r = 0; r < CPL; ++r) y[r] = 0.f;
    for (int aa = 0; aa < a.bw; ++aa) {
      const float xa = x[aa];
      if (xa == 0.f) continue;
      const float* kr = a.Kc + (int64_t)aa * a.ldk;
#pragma unroll
      for (int r = 0; r < CPL; ++r) {
        const int col = lane + 64 * r;
        if (col < a.bw) y[r] = fmaf(xa, kr[col], y[r]);
      }
    }
  };
  if (comp) {
    // right-hand side (w~ K)_k: w~ = the row's weights on the removed columns, zero elsewhere
#pragma unroll
    for (int r = 0; r < CPL; ++r) sm.key[lane + 64 * r] = sel[r] ? wv[r] : 0.f;
    WAVE_SYNC();
    float t[CPL];
    matvec_k(sm.key, t);
    if (ns == 0) {  // the whole block goes: lambda = w~ K
#pragma unroll
      for (int r = 0; r < CPL; ++r) {
        const int col = lane + 64 * r;
        if (col < a.bw) lam_g[col] = t[r];
      }
      return;
    }
#pragma unroll
    for (int r = 0; r < CPL; ++r) sm.wrow[lane + 64 * r] = t[r];  // gathered below through q
  }
  WAVE_SYNC();

  // ---- tile grid: nt tile rows, and the PARTIAL tile comes first.  Matrix index m < 32 - pad
  //      is unknown m, 32 - pad <= m < 32 is padding (identity, never eliminated), m >= 32 is
  //      unknown m - pad.  A pivot costs one MFMA per live tile, most in the first tile row
  //      (NTR (NTR + 1) / 2 of them): with the short tile row in front, a system of 66 unknowns
  //      costs 2 * 6 + 32 * 3 + 32 MFMAs instead of 32 * 6 + 32 * 3 + 2. ----
  const int nt = FULL ? NTR : (ns + 31) >> 5;
  const int pad = FULL ? 0 : 32 * nt - ns;
  auto valid = [&](int m) { return FULL || m < 32 - pad || (m >= 32 && m - pad < ns); };
  auto unk = [&](int m) {  // clamped: always a valid index
    return FULL ? m : min(m < 32 ? m : m - pad, ns - 1);
  };

  // ---- gather R_hat = G[q, q] into the tiles (all loads unconditional from clamped, valid
  //      indices, masked afterwards); right-hand side distributed by row ----
  const float* G = comp ? a.Kc : a.P + a.j1 * a.b + a.j1;  // R_hat = G[q, q], or K[k, k]
  const unsigned int bb = comp ? (unsigned int)a.ldk : (unsigned int)a.b;  // q * b < 2^31
  f32x16 T[NTR][NTR];
  unsigned int qcol[NTR];
#pragma unroll
  for (int ti = 0; ti < NTR; ++ti) qcol[ti] = sm.q[unk(32 * ti + lo)];
#pragma unroll
  for (int tj = 0; tj < NTR; ++tj) {
    if (tj < nt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + 4 * hi + (r & 3);  // tile row held in register r
        const unsigned int off = (unsigned int)sm.q[unk(32 * tj + row)] * bb;
#pragma unroll
        for (int ti = tj; ti < NTR; ++ti) T[ti][tj][r] = G[off + qcol[ti]];
      }
    }
  }
#pragma unroll
  for (int tj = 0; tj < NTR; ++tj)
#pragma unroll
    for (int ti = tj; ti < NTR; ++ti)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r >> 2) + 4 * hi + (r & 3);
        const float ident = (ti == tj && row == lo) ? 1.f : 0.f;  // identity outside the system
        T[ti][tj][r] = (tj < nt && ti < nt && valid(32 * tj + row) && valid(32 * ti + lo))
                           ? T[ti][tj][r] : ident;
      }
  // Each half of the wavefront only sees the pivots whose row it holds, so the value of a row of
  // the right-hand side is the SUM of its two lanes (lo and lo + 32); it starts in the lower half.
  float uv[NTR], zz[NZ];
#pragma unroll
  for (int ti = 0; ti < NTR; ++ti)
    uv[ti] = (hi == 0 && ti < nt && valid(32 * ti + lo)) ? sm.wrow[sm.q[unk(32 * ti + lo)]] : 0.f;
#pragma unroll
  for (int z = 0; z < NZ; ++z) zz[z] = 0.f;  // position 64 z + lane: y / d
  // Two pivots per MFMA: rows k1 and k2 = k1 + 4 (k1 mod 8 < 4) of a tile sit in the same
  // register, in the lower and in the upper half of the wavefront, where the two reduction slots
  // of v_mfma_f32_32x32x2_f32 take their operands.  The pivots of a tile are therefore taken in
  // the order 0,4,1,5,2,6,3,7,8,12,...; pair t = (k1, k2) holds POSITIONS 2t and 2t + 1 of that
  // order.  L~ (unit lower triangular in elimination order), z and lambda are indexed by
  // position; mrow() maps a position back to its matrix index.
  const int pl = 8 * (lo >> 3) + 2 * (lo & 3) + ((lo >> 2) & 1);  // position of index lo in a tile
  auto mrow = [](int P) { return (P & ~7) + ((P & 7) >> 1) + 4 * (P & 1); };
  // where this lane's element of a column of L~ goes: the packed row of its position; lanes
  // whose element is on / above the diagonal write to scratch
  float* rowp[NTR];
#pragma unroll
  for (int ti = 0; ti < NTR; ++ti) rowp[ti] = &sm.L[(32 * ti + pl) * (32 * ti + pl - 1) / 2];
  float* const junk = &sm.dummy[32 + lo];
  bool bad = false;

#pragma unroll
  for (int p = 0; p < NTR; ++p) {
    if (p < nt) {
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const int k1 = 8 * (t >> 2) + (t & 3), k2 = k1 + 4;
        if (p > 0 || k1 < 32 - pad) {  // a padding row paired with a real one is a no-op pivot
          const float v = T[p][p][t];   // lower half: row k1 of the reduced tile, upper half: row k2
          const float x = lower_half(v);
          const float d1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), k1));
          const float c12 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), k2));
          const float d2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32 + k2));
          const float y1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(uv[p]), k1)) +
                           __int_as_float(__builtin_amdgcn_readlane(__float_as_int(uv[p]), k1 + 32));
          const float y2r = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(uv[p]), k2)) +
                            __int_as_float(__builtin_amdgcn_readlane(__float_as_int(uv[p]), k2 + 32));
          const float q1 = __builtin_amdgcn_rcpf(d1);
          const float r1 = fmaf(fmaf(-d1, q1, 1.f), q1, q1);
          const float m = c12 * r1;
          const float d2p = fmaf(-c12, m, d2);  // pivot of k2 after the elimination of k1
          const float q2 = __builtin_amdgcn_rcpf(d2p);
          const float r2 = fmaf(fmaf(-d2p, q2, 1.f), q2, q2);
          const float y2 = fmaf(-m, y1, y2r);
          bad = bad || !(d1 > 0.f) || !(d2p > 0.f);
          const float mh = hi ? m : 0.f;
          const float rh = hi ? -r2 : -r1;
          const float yh = hi ? y2 : y1;
          // u1 (lower half) and u2 = row k2 after the elimination of k1 (upper half).  Columns
          // eliminated earlier hold rounding residue instead of zero; it is not masked, because
          // a product with it only ever lands in eliminated rows and columns of the tiles and in
          // right-hand-side rows that have already been read.
          const float bop = fmaf(-mh, x, v);
          const float aop = bop * rh;
          T[p][p] = __builtin_amdgcn_mfma_f32_32x32x2f32(aop, bop, T[p][p], 0, 0, 0);
          // column 2t + hi of L~ within the tile: rows at later positions
          (pl > 2 * t + hi ? rowp[p] + 32 * p + hi : junk)[2 * t] = -aop;
          uv[p] = fmaf(aop, yh, uv[p]);
          if ((lane >> 1) == (((32 * p + 2 * t) & 63) >> 1))
            zz[(32 * p + 2 * t) >> 6] = (lane & 1) ? y2 * r2 : y1 * r1;
          float e2[NTR], be[NTR];
#pragma unroll
          for (int ti = p + 1; ti < NTR; ++ti) {
            if (ti < nt) {
              // R_hat[32 ti + lo][32 p + k1] (lower half) and [..][32 p + k2] (upper half)
              const float ev = T[ti][p][t];
              const float xe = lower_half(ev);
              e2[ti] = fmaf(-mh, xe, ev);
              be[ti] = rh * e2[ti];
              T[ti][p] = __builtin_amdgcn_mfma_f32_32x32x2f32(bop, be[ti], T[ti][p], 0, 0, 0);
              (rowp[ti] + 32 * p + hi)[2 * t] = -be[ti];
              uv[ti] = fmaf(be[ti], yh, uv[ti]);
#pragma unroll
              for (int tj = p + 1; tj <= ti; ++tj) {
                // transposed storage: the first operand runs over the rows of tile row tj
                T[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x2f32(be[tj], e2[ti], T[ti][tj], 0, 0, 0);
              }
            }
          }
        }
      }
    }
  }
  if (bad && lane == 0) atomicCAS(a.info, 0, -(int32_t)min(i + 1, (int64_t)0x7fffffff));
  WAVE_SYNC();

  // ---- L~^T lambda = z: lambda_k is final once all rows below it are done; then column k of
  //      L~^T (= row k of L~, one LDS row) is swept out of the rows above.  The LDS rows of eight
  //      unknowns are fetched together, ahead of the dependent chain. ----
#pragma unroll
  for (int k8 = 32 * NTR - 8; k8 >= 0; k8 -= 8) {
    if (k8 < 32 * nt) {
      float row[8][NZ];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int k = k8 + t;
#pragma unroll
        for (int z = 0; z < NZ; ++z)  // lanes past the row read beyond it: masked below
          row[t][z] = (64 * z < k) ? sm.L[k * (k - 1) / 2 + 64 * z + lane] : 0.f;
      }
#pragma unroll
      for (int t = 7; t >= 0; --t) {
        const int k = k8 + t;
        if (k >= 1 && k < 32 * nt && valid(mrow(k))) {
          const float lk =
              __int_as_float(__builtin_amdgcn_readlane(__float_as_int(zz[k >> 6]), k & 63));
#pragma unroll
          for (int z = 0; z < NZ; ++z)
            if (64 * z < k) zz[z] = fmaf(-((64 * z + lane < k) ? row[t][z] : 0.f), lk, zz[z]);
        }
      }
    }
  }

  // ---- lambda row: zeros except lambda_l at column q_l ----
#pragma unroll
  for (int r = 0; r < CPL; ++r) sm.wrow[lane + 64 * r] = 0.f;
  WAVE_SYNC();
#pragma unroll
  for (int z = 0; z < NZ; ++z)
    if (64 * z + lane < 32 * nt && valid(mrow(64 * z + lane)))
      sm.wrow[sm.q[unk(mrow(64 * z + lane))]] = zz[z];
  WAVE_SYNC();
  if (comp) {
    // wrow holds y on the kept columns: lambda = ((w~ - y~) K)_q
#pragma unroll
    for (int r = 0; r < CPL; ++r)
      sm.key[lane + 64 * r] = (sel[r] ? wv[r] : 0.f) - sm.wrow[lane + 64 * r];
    WAVE_SYNC();
    float l[CPL];
    matvec_k(sm.key, l);
#pragma unroll
    for (int r = 0; r < CPL; ++r) {
      const int col = lane + 64 * r;
      if (col < a.bw) lam_g[col] = sel[r] ? l[r] : 0.f;
    }
    return;
  }
#pragma unroll
  for (int r = 0; r < CPL; ++r) {
    const int col = lane + 64 * r;
    if (col < a.bw) lam_g[col] = sm.wrow[col];
  }
}

// ------------------------------------------------------------------------------------------
// Mask + per-row solve for systems of 65..256 unknowns (block width <= 512): one workgroup of
// four or eight wavefronts per row of W.  R_hat = G[q, q] is held in LDS as the lower triangle of a grid
// of 32x32 tiles (padded with the identity past s) and factored by a right-looking blocked
// Cholesky, R_hat = L L^T, 32 columns per step:
//   1. one wavefront eliminates the diagonal tile with rank-1 MFMAs on its accumulator-layout
//      copy (row k of a symmetric tile is both operands of D -= u u^T / d; two pivots per
//      MFMA, see tl_pivots) and carries a second tile that starts as I along, which ends as
//      T = L_pp^{-1} for a factor L_pp L_pp^T of the tile; T replaces the diagonal tile;
//   2. the tiles below it become L_ip = A_ip T^T (one 32x32x32 product each), y_p = T u_p;
//   3. the tiles right of the panel get A_il -= L_ip L_lp^T, the right-hand side u_i -= L_ip y_p;
//      meanwhile one wavefront updates the next diagonal tile and runs step 1 on it (look-ahead:
//      the elimination is a chain of dependent instructions, the rest is throughput work).
// L^T lambda = y is then solved from the last tile row upwards with the same T tiles.
// All products are fp32 MFMAs (v_mfma_f32_32x32x2_f32) on operands read from LDS.
constexpr int kTlLd = 33;          // LDS row stride of a tile (conflict-free rows and columns)
constexpr int kTlSz = 32 * kTlLd;  // floats per tile
constexpr int kTlSmax = 256;       // largest system
constexpr int kTlBw = 512;         // widest block
constexpr int kTlExtra = 3 * kTlSmax + 128 + 16;  // u, lambda, q, pivot scratch, counters

__host__ __device__ inline int tl_ntiles(int nt) { return nt * (nt + 1) / 2; }
static inline size_t tl_smem_bytes(int nt) {
  return ((size_t)tl_ntiles(nt) * kTlSz + kTlExtra) * sizeof(float);
}
__device__ __forceinline__ int tl_row(int r, int hi) { return 8 * (r >> 2) + 4 * hi + (r & 3); }
__device__ __forceinline__ float* tl_tile(float* tiles, int i, int j) {
  return tiles + (i * (i + 1) / 2 + j) * kTlSz;
}
// acc += sign * A * Bn^T for 32x32 tiles, A[m][k] at pa[m*kTlLd + k], Bn[n][k] at pb[n*kTlLd + k]
__device__ __forceinline__ void tl_mma(f32x16& acc, const float* pa, const float* pb, float sign,
                                       int lo, int hi) {
  float av[16], bv[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    av[e] = pa[lo * kTlLd + 2 * e + hi];
    bv[e] = pb[lo * kTlLd + 2 * e + hi];
  }
#pragma unroll
  for (int e = 0; e < 16; ++e)
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(sign * av[e], bv[e], acc, 0, 0, 0);
}
// Eliminates the symmetric tile D (accumulator layout) and writes T = F^{-1}, F F^T = D, to Dt.
// One wavefront.  Returns true if a pivot was not positive.
//
// Two pivots per MFMA.  In the accumulator layout rows k and k + 4 (k mod 8 < 4) sit in the same
// register, in the lower and in the upper half of the wavefront: exactly where the two
// reduction slots of v_mfma_f32_32x32x2_f32 take their operands from.  The pivots are therefore
// taken in the order 0,4,1,5,2,6,3,7,8,12,...: with u1 = row k and u2 = row k + 4 AFTER the
// elimination of k (u2 = D[k+4] - (D[k][k+4] / d1) u1; the lower half's row is fetched with one
// cross-lane read), D -= u1 u1^T / d1 + u2 u2^T / d2 is one MFMA instead of two half-empty
// ones.  The same row operations applied to a tile that starts as I give T~; F is the Cholesky
// factor in that pivot order (a row-permuted triangle).  Nothing downstream needs a triangle:
// the panel products, the substitutions and the trailing updates only use T as a dense tile.
__device__ __forceinline__ bool tl_pivots(f32x16 D, float* Dt, float* aux, int lo, int hi) {
  f32x16 E;
#pragma unroll
  for (int r = 0; r < 16; ++r) E[r] = (tl_row(r, hi) == lo) ? 1.f : 0.f;
  const int pidx = 4 * (lo >> 3) + (lo & 3);  // pair that eliminates column lo
  float dl = 1.f;                             // pivot of column lo
#pragma unroll
  for (int t = 0; t < 16; ++t) {              // pair t: rows k1 and k2 = k1 + 4, both in D[t]
    const int k1 = 8 * (t >> 2) + (t & 3), k2 = k1 + 4;
    const float v = D[t];                     // lower half: D[k1][lo], upper half: D[k2][lo]
    const float x = lower_half(v);        // D[k1][lo] in both halves
    const float d1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), k1));
    const float c12 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), k2));
    const float d2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32 + k2));
    // 1 / d1 and 1 / d2' (d2' = d2 - c12^2 / d1, the pivot of k2 after the elimination of k1)
    // from two INDEPENDENT reciprocals, of d1 and of det = d1 d2 - c12^2: d2' = det / d1.  The
    // wavefront is alone on this chain, so its length is what counts.
    const float det = fmaf(d1, d2, -c12 * c12);
    const float q1 = __builtin_amdgcn_rcpf(d1);
    const float qd = __builtin_amdgcn_rcpf(det);
    const float r1 = fmaf(fmaf(-d1, q1, 1.f), q1, q1);
    const float rd = fmaf(fmaf(-det, qd, 1.f), qd, qd);
    const float m = c12 * r1;
    const float d2p = det * r1;
    const float r2 = d1 * rd;
    const float mh = hi ? m : 0.f;
    // second operands: u1 in the lower half, u2 in the upper half; columns eliminated by
    // earlier pairs are zero, and so is column k1 of u2
    const bool live = pidx >= t && !(hi && lo == k1);
    const float bop = live ? fmaf(-mh, x, v) : 0.f;
    const float aop = bop * (hi ? -r2 : -r1);
    D = __builtin_amdgcn_mfma_f32_32x32x2f32(aop, bop, D, 0, 0, 0);
    dl = (lo == k1) ? d1 : (lo == k2) ? d2p : dl;
    // the same row operations on T~: row k1 as it is, row k2 after the operation of k1; the
    // pivot rows themselves stay
    const float ev = E[t];
    const float xe = lower_half(ev);
    const float be = fmaf(-mh, xe, ev);
    const float a2 = (lo == (hi ? k2 : k1)) ? 0.f : aop;
    E = __builtin_amdgcn_mfma_f32_32x32x2f32(a2, be, E, 0, 0, 0);
  }
  const bool bad = __ballot(!(dl > 0.f)) != 0ull;
  float isd = __builtin_amdgcn_rsqf(dl);
  isd = fmaf(0.5f * isd, fmaf(-dl * isd, isd, 1.f), isd);
  aux[lo] = isd;  // both halves write the same value
#pragma unroll
  for (int r = 0; r < 16; ++r)  // F^{-1} = diag(1/sqrt(d)) T~
    Dt[tl_row(r, hi) * kTlLd + lo] = E[r] * aux[tl_row(r, hi)];
  return bad;
}

// y[j] = sum_a x[a] * K[a * ldk + j], j < bw (bw a multiple of 4, K 16-byte aligned rows), for a
// workgroup of NW wavefronts; x and y in LDS.  Rows with x[a] == 0 are skipped (uniform test).
// !BIG (bw <= 512): the wavefronts split the rows a, each lane holds up to two groups of four
// columns, partial sums meet in part[NW][bw] (LDS) and are added in a fixed order.
// BIG: every wavefront owns column groups and walks all rows; no partial sums.
// Barriers inside; x must be complete on entry, y is complete on return.
template <int NW, bool BIG>
__device__ __forceinline__ void tl_matvec(const float* x, int bw, const float* __restrict__ K,
                                          int ldk, float* y, float* part) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ng = bw >> 2;
  if (BIG) {
    for (int g = 64 * wave + lane; g < ng; g += 64 * NW) {
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
      for (int a = 0; a < bw; ++a) {
        const float xa = x[a];
        const float4 k4 = *reinterpret_cast<const float4*>(K + (int64_t)a * ldk + 4 * g);
        acc.x = fmaf(xa, k4.x, acc.x);
        acc.y = fmaf(xa, k4.y, acc.y);
        acc.z = fmaf(xa, k4.z, acc.z);
        acc.w = fmaf(xa, k4.w, acc.w);
      }
      *reinterpret_cast<float4*>(y + 4 * g) = acc;
    }
    __syncthreads();
    return;
  }
  const int per = (bw + NW - 1) / NW;
  const int alo = wave * per, ahi = min(bw, alo + per);
  float4 acc[2] = {make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f)};
  const int g0 = min(lane, ng - 1), g1 = min(lane + 64, ng - 1);  // clamped: loads stay in bounds
#pragma unroll 4
  for (int a = alo; a < ahi; ++a) {
    const float xa = x[a];
    if (xa == 0.f) continue;
    const float4 k0 = *reinterpret_cast<const float4*>(K + (int64_t)a * ldk + 4 * g0);
    const float4 k1 = *reinterpret_cast<const float4*>(K + (int64_t)a * ldk + 4 * g1);
    acc[0].x = fmaf(xa, k0.x, acc[0].x);
    acc[0].y = fmaf(xa, k0.y, acc[0].y);
    acc[0].z = fmaf(xa, k0.z, acc[0].z);
    acc[0].w = fmaf(xa, k0.w, acc[0].w);
    acc[1].x = fmaf(xa, k1.x, acc[1].x);
    acc[1].y = fmaf(xa, k1.y, acc[1].y);
    acc[1].z = fmaf(xa, k1.z, acc[1].z);
    acc[1].w = fmaf(xa, k1.w, acc[1].w);
  }
  if (lane < ng) *reinterpret_cast<float4*>(part + wave * bw + 4 * lane) = acc[0];
  if (lane + 64 < ng) *reinterpret_cast<float4*>(part + wave * bw + 4 * (lane + 64)) = acc[1];
  __syncthreads();
  for (int j = tid; j < bw; j += 64 * NW) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += part[w * bw + j];
    y[j] = t;
  }
  __syncthreads();
}

// BIG = false: tiles in LDS, one workgroup per row (grid = c), systems of up to 256 unknowns in
// blocks of up to 512 columns.  BIG = true: the same algorithm for systems of up to kBigSmax
// unknowns in blocks of up to kBigBw columns (the large blocks of the paper's block-size
// ablation): the tile grid of a row no longer fits LDS and lives in global memory, one slot per
// workgroup (a.tile_scratch, a.slot_floats; the slot of a workgroup stays in the caches of its
// compute unit's XCD), and the gridDim.x workgroups walk the rows (row = blockIdx.x,
// blockIdx.x + gridDim.x, ...).  The row's right-hand side, multipliers, indices and the
// block's weights stay in LDS.
constexpr int kBigSmax = 2048;
constexpr int kBigBw = 4096;
static inline size_t tl_big_smem_bytes() {
  return ((size_t)2 * kBigBw + 3 * kBigSmax + 128 + 2 * 8 * (kBigBw / 512)) * sizeof(float);
}

template <int SEL, int NW, bool BIG = false>
__global__ __launch_bounds__(64 * NW, (BIG ? 2 : (NW == 8 ? 4 : 3))) void k_solve_tiled(SolveArgs a) {
  constexpr int NT = 64 * NW;       // threads
  constexpr int SMAX = BIG ? kBigSmax : kTlSmax;
  constexpr int BW = BIG ? kBigBw : kTlBw;
  constexpr int CH = BW / NT;       // block columns per thread
  constexpr int RPT = 1024 / NT;    // tile elements per thread
  constexpr int NC = NW * CH;       // (wavefront, column chunk) pairs
  extern __shared__ __attribute__((aligned(16))) char solve_smem[];
  float* tiles;
  float *wrow, *key, *xtra;
  if (BIG) {
    tiles = a.tile_scratch + (int64_t)blockIdx.x * a.slot_floats;
    wrow = reinterpret_cast<float*>(solve_smem);
    key = wrow + BW;
    xtra = key + BW;
  } else {
    tiles = reinterpret_cast<float*>(solve_smem);
    xtra = tiles + tl_ntiles(a.nt_max) * kTlSz;
    // the block's weights and metric live in the tile area until the gather overwrites them, and
    // the lambda row is assembled there after the solve (nt_max >= 3: room for 2 * kTlBw floats)
    wrow = tiles;
    key = tiles + BW;
  }
  float* u = xtra;                    // right-hand side, then y
  float* lam = xtra + SMAX;
  int* q = reinterpret_cast<int*>(xtra + 2 * SMAX);
  float* aux = xtra + 3 * SMAX;
  int* cnt = reinterpret_cast<int*>(aux + 128);  // per wavefront and chunk: selected, ties
  int* eqc = cnt + NC;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lo = lane & 31, hi = lane >> 5;
  for (int64_t i = blockIdx.x; i < a.c; i += gridDim.x) {  // !BIG: gridDim.x == c, one pass
  if (BIG) __syncthreads();  // the previous row's LDS and slot contents are dead
  const float* wrow_g = a.W + i * a.b + a.j1;

  // ---- selection of the block mask row M_i: column col = tid + NT * ch ----
  bool sel[CH];
  float wv[CH];
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    const int col = tid + NT * ch;
    wv[ch] = (col < a.bw) ? wrow_g[col] : 0.f;
    wrow[col] = wv[ch];
    sel[ch] = false;
  }
  if (SEL == SEL_GIVEN) {
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int col = tid + NT * ch;
      sel[ch] = (col < a.bw) && a.mask_in[i * a.b + a.j1 + col] != 0;
    }
  } else if (SEL == SEL_NM) {
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int col = tid + NT * ch;
      key[col] = (col < a.bw) ? fabsf(wv[ch]) * a.sx[a.j1 + col] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int col = tid + NT * ch;
      if (col < a.bw) {
        const int g0 = (col / a.m) * a.m;
        const float mine = key[col];
        int rank = 0;
        for (int e = 0; e < a.m; ++e) {
          const float o = key[g0 + e];
          rank += (o < mine || (o == mine && g0 + e < col)) ? 1 : 0;
        }
        sel[ch] = rank < a.n;
      }
    }
    if (a.row_skip && a.row_skip[i]) {
#pragma unroll
      for (int ch = 0; ch < CH; ++ch) sel[ch] = false;
    }
  } else {  // SEL_THRESHOLD: key < tau, or key == tau and among the first need_eq ties
    const bool none = a.st->none != 0;
    const unsigned int tau = a.st->tau;
    const long long need_eq = a.st->need_eq;
    bool lt[CH], eq[CH];
    unsigned long long eqb[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int col = tid + NT * ch;
      const bool in = (col < a.bw) && !none;
      const unsigned int kk = in ? metric_key(wv[ch], a.sx[a.j1 + col]) : 0xffffffffu;
      lt[ch] = in && kk < tau;
      eq[ch] = in && kk == tau;
      eqb[ch] = __ballot(eq[ch]);
      if (lane == 0) eqc[NW * ch + wave] = __popcll(eqb[ch]);
    }
    __syncthreads();
    const long long ties0 = ties_before(a.st, a.row_eq, i);
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      long long my = ties0;
      for (int v = 0; v < NW * ch + wave; ++v) my += eqc[v];
      my += __popcll(eqb[ch] & ((1ull << lane) - 1ull));
      sel[ch] = lt[ch] || (eq[ch] && my < need_eq);
    }
  }

  // ---- q = phi(M_i) (ascending column indices) and s ----
  unsigned long long bal[CH];
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    bal[ch] = __ballot(sel[ch]);
    if (lane == 0) cnt[NW * ch + wave] = __popcll(bal[ch]);
  }
  __syncthreads();
  int s = 0;
#pragma unroll
  for (int v = 0; v < NC; ++v) s += cnt[v];
  // A row that loses more than half of the block is solved through the complement: with
  // K = G^{-1}, kept set k of the block and w~ = (u on q, 0 on k),
  //     (G_qq)^{-1} = K_qq - K_qk (K_kk)^{-1} K_kq,   so   lambda = ((w~ - y~) K)_q
  // with y~ = (0 on q, y on k), y K_kk = (w~ K)_k: a system of bw - s unknowns instead of s,
  // and never more than half a block.  (Same accuracy: K is formed from the factor directly.)
  const bool comp = a.Kc != nullptr && 2 * s > a.bw;  // uniform per workgroup
  const int ns = comp ? a.bw - s : s;                  // unknowns of this row's system
  if (SEL == SEL_THRESHOLD) {
    if (tid == 0) a.row_cnt[i] = s;  // summed at the start of the next block
  }
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    const int col = tid + NT * ch;
    if (col < a.bw) a.mask_out[i * a.b + a.j1 + col] = sel[ch] ? 1 : 0;
  }
  // A block may be solved by two launches with different LDS footprints: this one takes the
  // rows with nt_lo <= ceil(ns/32) <= nt_max and leaves the others untouched.
  const int nt = (ns + 31) >> 5;
  const bool fits = ns <= SMAX;
  if (fits ? (nt < a.nt_lo || nt > a.nt_max) : (32 * a.nt_max < SMAX)) {
    if (BIG) continue;
    return;
  }
  // the solved set: removed columns, or kept columns of the block when solving the complement
  bool ins[CH];
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) ins[ch] = comp ? (tid + NT * ch < a.bw && !sel[ch]) : sel[ch];
  if (comp) {
    __syncthreads();  // all counts of the removed set have been read
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      bal[ch] = __ballot(ins[ch]);
      if (lane == 0) cnt[NW * ch + wave] = __popcll(bal[ch]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int ch = 0; ch < CH; ++ch) {
    const int col = tid + NT * ch;
    int before = 0;
    for (int v = 0; v < NW * ch + wave; ++v) before += cnt[v];
    if (ins[ch] && fits) q[before + __popcll(bal[ch] & ((1ull << lane) - 1ull))] = col;
  }
  float* lam_g = a.Lam + i * a.ldl;
  if (s == 0 || !fits) {  // !fits cannot happen for a launch chosen by the host
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int col = tid + NT * ch;
      if (col < a.bw) lam_g[col] = 0.f;
    }
    if (!fits && tid == 0) atomicCAS(a.info, 0, -(int32_t)min(i + 1, (int64_t)0x7fffffff));
    if (BIG) continue;
    return;
  }
  __syncthreads();
  // partial sums of the complement's matrix-vector products: behind wrow and key in the tile
  // area (nt_max >= 3: 6 tiles = 6336 floats >= 2 * 512 + 8 * 512)
  float* part = BIG ? nullptr : tiles + 2 * BW;
  if (!comp) {
    for (int t = tid; t < 32 * nt; t += NT) u[t] = (t < s) ? wrow[q[t]] : 0.f;
  } else {
    // right-hand side (w~ K)_k: x = w~ in `key`, the product lands in `wrow` (the row's weights
    // stay in registers)
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) key[tid + NT * ch] = sel[ch] ? wv[ch] : 0.f;
    __syncthreads();
    tl_matvec<NW, BIG>(key, a.bw, a.Kc, a.ldk, wrow, part);
    for (int t = tid; t < 32 * nt; t += NT) u[t] = (t < ns) ? wrow[q[t]] : 0.f;
  }
  __syncthreads();  // !BIG: wrow and key are dead from here on

  // ---- gather R_hat into the tiles: thread <-> (rows tid/32 + (NT/32)e, column tid%32) of a tile;
  //      up to four tiles of a tile row are fetched together, all loads unconditional from
  //      clamped (valid) indices and masked when stored ----
  if (ns > 0) {
    // R_hat = G[q, q], or K[k, k] for the complement
    const float* G = comp ? a.Kc : a.P + a.j1 * a.b + a.j1;
    const int64_t ldg = comp ? (int64_t)a.ldk : a.b;
    const int tr = tid >> 5, tc = tid & 31;
    for (int ti = 0; ti < nt; ++ti) {
      const float* grow[RPT];
#pragma unroll
      for (int e = 0; e < RPT; ++e)
        grow[e] = G + (int64_t)q[min(32 * ti + tr + (NT / 32) * e, ns - 1)] * ldg;
      for (int tj0 = 0; tj0 <= ti; tj0 += 4) {
        float v[4][RPT];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int tj = min(tj0 + t, ti);
          const int qc = q[min(32 * tj + tc, ns - 1)];
#pragma unroll
          for (int e = 0; e < RPT; ++e) v[t][e] = grow[e][qc];
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int tj = tj0 + t;
          if (tj <= ti) {
            float* T = tl_tile(tiles, ti, tj);
            const int cc = 32 * tj + tc;
#pragma unroll
            for (int e = 0; e < RPT; ++e) {
              const int rr = 32 * ti + tr + (NT / 32) * e;
              const float ident = (rr == cc) ? 1.f : 0.f;
              T[(tr + (NT / 32) * e) * kTlLd + tc] = (rr < ns && cc < ns) ? v[t][e] : ident;
            }
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- blocked Cholesky with look-ahead, forward substitution carried along.  The wavefront
  //      that eliminates a diagonal tile rotates, so that concurrent workgroups of a compute
  //      unit do not run this latency-bound step on the same SIMD. ----
  bool bad = false;
  if (nt > 0 && wave == ((int)blockIdx.x & (NW - 1))) {
    f32x16 D;
#pragma unroll
    for (int r = 0; r < 16; ++r) D[r] = tiles[tl_row(r, hi) * kTlLd + lo];
    bad = tl_pivots(D, tiles, aux, lo, hi);
  }
  __syncthreads();
  for (int p = 0; p < nt; ++p) {
    float* Tp = tl_tile(tiles, p, p);
    {  // panel: L_ip = A_ip T^T
      for (int ii = p + 1 + wave; ii < nt; ii += NW) {
        float* Aip = tl_tile(tiles, ii, p);
        f32x16 C;
#pragma unroll
        for (int r = 0; r < 16; ++r) C[r] = 0.f;
        tl_mma(C, Aip, Tp, 1.f, lo, hi);
#pragma unroll
        for (int r = 0; r < 16; ++r) Aip[tl_row(r, hi) * kTlLd + lo] = C[r];
      }
      if (wave == NW - 1 && lane < 32) {  // y_p = T u_p
        float acc = 0.f;
#pragma unroll
        for (int k = 0; k < 32; ++k) acc = fmaf(Tp[lane * kTlLd + k], u[32 * p + k], acc);
        u[32 * p + lane] = acc;
      }
    }
    __syncthreads();
    if (p + 1 == nt) break;
    // One wavefront brings the next diagonal tile up to date and eliminates it at once (the
    // tile stays in registers); the others apply panel p to the rest of the trailing
    // matrix, the tiles of column p+1 first, and to the right-hand side.
    const int pw = (p + 1 + (int)blockIdx.x) & (NW - 1);
    if (wave == pw) {
      float* Dn = tl_tile(tiles, p + 1, p + 1);
      const float* Lp = tl_tile(tiles, p + 1, p);
      f32x16 D;
#pragma unroll
      for (int r = 0; r < 16; ++r) D[r] = Dn[tl_row(r, hi) * kTlLd + lo];
      tl_mma(D, Lp, Lp, -1.f, lo, hi);
      bad = tl_pivots(D, Dn, aux, lo, hi) || bad;
    } else {
      const int widx = wave - (wave > pw ? 1 : 0);  // 0..NW-2
      int t = 0, mine = widx;
      auto upd = [&](int ii, int l) {
        float* Ail = tl_tile(tiles, ii, l);
        f32x16 C;
#pragma unroll
        for (int r = 0; r < 16; ++r) C[r] = Ail[tl_row(r, hi) * kTlLd + lo];
        tl_mma(C, tl_tile(tiles, ii, p), tl_tile(tiles, l, p), -1.f, lo, hi);
#pragma unroll
        for (int r = 0; r < 16; ++r) Ail[tl_row(r, hi) * kTlLd + lo] = C[r];
      };
      for (int ii = p + 2; ii < nt; ++ii, ++t)
        if (t == mine) {
          upd(ii, p + 1);
          mine += NW - 1;
        }
      for (int l = p + 2; l < nt; ++l)
        for (int ii = l; ii < nt; ++ii, ++t)
          if (t == mine) {
            upd(ii, l);
            mine += NW - 1;
          }
      for (int row = 32 * (p + 1) + 64 * widx + lane; row < 32 * nt; row += 64 * (NW - 1)) {
        // u_i -= L_ip y_p
        const float* Lr = tl_tile(tiles, row >> 5, p) + (row & 31) * kTlLd;
        float acc = u[row];
#pragma unroll
        for (int k = 0; k < 32; ++k) acc = fmaf(-Lr[k], u[32 * p + k], acc);
        u[row] = acc;
      }
    }
    __syncthreads();
  }
  if (bad && lane == 0) atomicCAS(a.info, 0, -(int32_t)min(i + 1, (int64_t)0x7fffffff));

  // ---- L^T lambda = y, last tile row first ----
  for (int p = nt - 1; p >= 0; --p) {
    const float* Tp = tl_tile(tiles, p, p);
    if (wave == 0 && lane < 32) {  // lambda_p = T^T y_p
      float acc = 0.f;
#pragma unroll
      for (int k = 0; k < 32; ++k) acc = fmaf(Tp[k * kTlLd + lane], u[32 * p + k], acc);
      lam[32 * p + lane] = acc;
    }
    __syncthreads();
    for (int t = tid; t < 32 * p; t += NT) {  // y_j -= L_pj^T lambda_p for the tile rows above
      const float* Lc = tl_tile(tiles, p, t >> 5) + (t & 31);
      float acc = u[t];
#pragma unroll
      for (int r = 0; r < 32; ++r) acc = fmaf(-Lc[r * kTlLd], lam[32 * p + r], acc);
      u[t] = acc;
    }
    __syncthreads();
  }

  // ---- lambda row: zeros except lambda_k at column q_k ----
  if (!comp) {
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) wrow[tid + NT * ch] = 0.f;
    __syncthreads();
    for (int t = tid; t < s; t += NT) wrow[q[t]] = lam[t];
    __syncthreads();
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int col = tid + NT * ch;
      if (col < a.bw) lam_g[col] = wrow[col];
    }
  } else {
    // lambda = ((w~ - y~) K)_q: x = w on the removed columns, -y on the kept ones
    __syncthreads();
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) key[tid + NT * ch] = sel[ch] ? wv[ch] : 0.f;
    __syncthreads();
    for (int t = tid; t < ns; t += NT) key[q[t]] = -lam[t];
    __syncthreads();
    tl_matvec<NW, BIG>(key, a.bw, a.Kc, a.ldk, wrow, part);
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
      const int col = tid + NT * ch;
      if (col < a.bw) lam_g[col] = sel[ch] ? wrow[col] : 0.f;
    }
  }
  if (!BIG) return;  // one row per workgroup
  }  // rows of this workgroup
}

// ------------------------------------------------------------------------------------------
// W[:, j1:b] -= Lam * P[j1:j2, j1:b]; removed weights of the block become exact zeros.
// W[:, col0:col_end] -= Lam[:, 0:K] * P[prow0:prow0+K, col0:col_end]; entries of the column
// range [zj1, zj2) whose mask byte is set are written as exact zeros.
struct UpdateArgs {
  float* W;
  const float* Lam;     // c x K multipliers, row stride ldl
  const float* P;
  const uint8_t* mask;
  int64_t c, b;
  int64_t prow0;        // first row of P (= first reduction index)
  int64_t col0, col_end;
  int64_t zj1, zj2;
  int K, ldl, vec_a, vec_b;
  int vec_w;            // W 8-byte and mask 2-byte aligned, b and col0 even: row pass in pairs
  // Unstructured mode: while the new weights are at hand, the columns right of the block are
  // histogrammed for the NEXT block's selection (window around the current threshold, see
  // k_select); hist == nullptr switches this off.
  unsigned int* hist;         // 2048 bins, global
  unsigned int* below_part;   // keys below the window, one count per workgroup
  unsigned int* cand_n;       // per workgroup: keys inside the window ...
  uint2* cand;                // ... and the keys with their rows, kCandStage slots per workgroup
  SelState* st;
  const float* sx;
  int gx, gy;                 // tile grid (set by launch_update)
};

constexpr size_t kUpdSmemBytes = kXSmemBytes + 2048 * sizeof(unsigned int) +
                                 16 * sizeof(unsigned int) + kCandStage * sizeof(uint2);

__global__ __launch_bounds__(kXThreads, 4) void k_update(UpdateArgs a) {
  extern __shared__ __attribute__((aligned(16))) char sm[];
  if (threadIdx.x == 0) TL_MARK(0);
  unsigned int* hw = reinterpret_cast<unsigned int*>(sm + kXSmemBytes);  // window histogram
  unsigned int* nb_wave = hw + 2048;  // 8 counts per wavefront, then: staged keys, list offset
  uint2* stage = reinterpret_cast<uint2*>(nb_wave + 16);
  // Tile of this workgroup.  Consecutive workgroup ids go to the eight XCDs in turn, each with
  // an L2 of its own: XCD x takes the row tiles x*rp .. x*rp + rp - 1 and walks them column by
  // column, so that it reads one eighth of the multipliers and every tile of P_k once.
  // (With fewer than 16 row tiles the XCDs would not get equal shares: plain order.)
  int bx, by;
  if (a.gy >= 16) {
    const int rp = (a.gy + 7) >> 3;
    const int slot = (int)blockIdx.x >> 3;
    bx = slot / rp;
    by = ((int)blockIdx.x & 7) * rp + (slot - bx * rp);
    if (by >= a.gy) return;
  } else {
    by = (int)blockIdx.x / a.gx;
    bx = (int)blockIdx.x - by * a.gx;
  }
  const int64_t m0 = (int64_t)by * kTM;
  const int64_t n0 = a.col0 + (int64_t)bx * kTN;
  const int m_ext = (int)min((int64_t)kTM, a.c - m0);
  const int n_ext = (int)min((int64_t)kTN, a.col_end - n0);
  const float* A = a.Lam + m0 * a.ldl;          // (m,k) at A[m*ldl + k]
  const float* Bm = a.P + a.prow0 * a.b + n0;   // (k,n) at B[k*b + n]
  // does this tile feed the next selection?  (uniform per workgroup)
  const bool win = a.hist != nullptr && !a.st->none && a.st->pred_try && n0 + n_ext > a.zj2;
  if (win) {
    for (int e = threadIdx.x; e < 2048; e += kXThreads) hw[e] = 0u;  // barriers follow in the product
    if (threadIdx.x == 0) nb_wave[8] = 0u;                            // staged keys
  }
  TileAcc acc;
  acc_zero(acc);
  gemm_tile_x3<false, true>(acc, sm, A, a.ldl, m_ext, Bm, a.b, n_ext, 0, a.K, a.vec_a, a.vec_b);
  if (threadIdx.x == 0) TL_MARK(1);
  const float* T = x3_stage_tile(acc, sm);
  if (threadIdx.x == 0) TL_MARK(2);
  // row pass: wavefront w takes rows w, w + 8, ..., lane l the columns 2l, 2l + 1
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = 2 * lane;
  const int64_t cg = n0 + c0;
  const bool in_block = n0 < a.zj2 && n0 + kTN > a.zj1;  // tile overlaps the columns holding masks
  float* Wg = a.W + m0 * a.b + cg;
  const uint8_t* Mg = a.mask + m0 * a.b + cg;
  // window count of one new weight (columns right of the block only)
  const unsigned int wlo = win ? a.st->win_lo : 0u;
  const int wsh = win ? a.st->win_shift : kWinShiftMin;
  unsigned int nb = 0;
  auto count = [&](float w, float sxj, int row) {
    const unsigned int key = metric_key(w, sxj);
    const unsigned int p28 = key >> wsh;
    if (p28 < wlo) {
      ++nb;
    } else if (p28 - wlo < 2048u) {
      atomicAdd(&hw[p28 - wlo], 1u);
      const unsigned int k = atomicAdd(&nb_wave[8], 1u);
      if (k < (unsigned int)kCandStage) stage[k] = make_uint2(key, (unsigned int)(m0 + row));
    }
  };
  if (m_ext == kTM && n_ext == kTN && a.vec_w) {  // whole tile, aligned pairs
    const bool z0 = in_block && cg >= a.zj1 && cg < a.zj2;
    const bool z1 = in_block && cg + 1 >= a.zj1 && cg + 1 < a.zj2;
    const bool h0 = win && cg >= a.zj2, h1 = win && cg + 1 >= a.zj2;
    const float sx0 = h0 ? a.sx[cg] : 0.f, sx1 = h1 ? a.sx[cg + 1] : 0.f;
    float2 old[16];
    unsigned short mk[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int64_t off = (int64_t)(wave + 8 * i) * a.b;
      old[i] = *reinterpret_cast<const float2*>(Wg + off);
      mk[i] = in_block ? *reinterpret_cast<const unsigned short*>(Mg + off) : (unsigned short)0;
    }
    TL_WAIT_LOADS();
    if (threadIdx.x == 0) TL_MARK(3);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = wave + 8 * i;
      const float2 t = *reinterpret_cast<const float2*>(T + row * kXCLd + c0);
      float2 o;
      o.x = (z0 && (mk[i] & 0xffu)) ? 0.f : old[i].x - t.x;
      o.y = (z1 && (mk[i] >> 8)) ? 0.f : old[i].y - t.y;
      *reinterpret_cast<float2*>(Wg + (int64_t)row * a.b) = o;
      if (h0) count(o.x, sx0, row);
      if (h1) count(o.y, sx1, row);
    }
  } else {
    for (int i = 0; i < 16; ++i) {
      const int row = wave + 8 * i;
      if (row >= m_ext) break;
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        if (c0 + e < n_ext) {
          const int64_t off = (int64_t)row * a.b + e;
          const bool z = in_block && cg + e >= a.zj1 && cg + e < a.zj2 && Mg[off] != 0;
          const float o = z ? 0.f : Wg[off] - T[row * kXCLd + c0 + e];
          Wg[off] = o;
          if (win && cg + e >= a.zj2) count(o, a.sx[cg + e], row);
        }
      }
    }
  }
  if (threadIdx.x == 0) TL_MARK(4);
  if (a.hist == nullptr) {
    if (threadIdx.x == 0) TL_MARK(5);
    return;
  }
  // one partial count of the keys below the window per workgroup (summed by k_select:
  // thousands of atomics on one address would cost more than the pass), window bins by atomics
  for (int off = 32; off > 0; off >>= 1) nb += __shfl_down(nb, off, 64);
  if (lane == 0) nb_wave[wave] = nb;
  __syncthreads();
  const int tile = by * a.gx + bx;
  if (threadIdx.x == 0) {
    unsigned int t = 0;
    for (int v = 0; v < kXThreads / 64; ++v) t += nb_wave[v];
    a.below_part[tile] = t;
    unsigned int n = win ? nb_wave[8] : 0u;
    if (n > (unsigned int)kCandStage) {  // more window keys than a list holds: no prediction
      a.st->cand_overflow = 1;
      n = 0u;
    }
    a.cand_n[tile] = n;
  }
  if (blockIdx.x == 0) {
    // between two launches of k_select: the histograms of its radix passes and its counters
    for (int e = threadIdx.x; e < 3 * 2048; e += kXThreads) a.hist[2048 + e] = 0u;
    if (threadIdx.x == 0) a.st->arrived = a.st->nbin = a.st->bar = 0u;
  }
  if (!win) {
    if (threadIdx.x == 0) TL_MARK(5);
    return;
  }
  const unsigned int n = min(nb_wave[8], (unsigned int)kCandStage);
  uint2* list = a.cand + (size_t)tile * kCandStage;
  for (unsigned int e = threadIdx.x; e < n; e += kXThreads) list[e] = stage[e];
  for (int e = threadIdx.x; e < 2048; e += kXThreads)
    if (hw[e]) atomicAdd(&a.hist[e], hw[e]);
  if (threadIdx.x == 0) TL_MARK(5);
}

// ------------------------------------------------------------------------------------------
// Outlier rows (App. G.4.4 / Sec. 4.7): h_i = ||W_i X||^2 = W_i H W_i^T; the ceil(alpha c) rows
// with the largest h are left untouched.
// W_i H W_i^T = 2 sum_n W_in sum_{k >= n} W_ik Hl_kn with Hl = the lower triangle of H with its
// diagonal halved and zeros above it: the product T = W Hl only needs the reduction range
// k >= n of every output column, i.e. half of the full product.
__global__ __launch_bounds__(256) void k_lower_half_diag(const float* __restrict__ H, int64_t b,
                                                         float* __restrict__ Hl) {
  const int64_t i = blockIdx.y;
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= b) return;
  const float v = (j <= i) ? H[i * b + j] : 0.f;
  Hl[i * b + j] = (j == i) ? 0.5f * v : v;
}

// h[i] = 2 sum_j T[i][j] * W[i][j]; one wavefront per row, fp64 sum in a fixed order.
__global__ __launch_bounds__(256) void k_rowdot(const float* __restrict__ T,
                                                const float* __restrict__ W, int64_t c, int64_t b,
                                                float* __restrict__ h) {
  const int lane = threadIdx.x & 63;
  const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (i >= c) return;
  double acc = 0.0;
  for (int64_t j = lane; j < b; j += 64) acc += (double)T[i * b + j] * (double)W[i * b + j];
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
  if (lane == 0) h[i] = (float)(2.0 * acc);
}

// skip[i] = 1 for the n_out rows with the largest (h, row) (ascending order, ties by row index).
__global__ __launch_bounds__(256) void k_row_rank(const float* __restrict__ h, int64_t c,
                                                  int64_t n_out, uint8_t* __restrict__ skip) {
  __shared__ float hs[2048];  // competitors, one chunk at a time
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const float mine = (i < c) ? h[i] : 0.f;
  int64_t rank = 0;
  for (int64_t k0 = 0; k0 < c; k0 += 2048) {
    const int nk = (int)min((int64_t)2048, c - k0);
    __syncthreads();
    for (int e = threadIdx.x; e < nk; e += 256) hs[e] = h[k0 + e];
    __syncthreads();
    for (int e = 0; e < nk; ++e) {
      const float o = hs[e];
      rank += (o < mine || (o == mine && k0 + e < i)) ? 1 : 0;
    }
  }
  if (i < c) skip[i] = rank >= c - n_out ? 1 : 0;
}

// skip[i] = 1 for the n_out rows of W (c x b fp32) with the largest loss W_i H W_i^T (H: lower
// triangle).  Hf (b x b, receives the lower triangle with halved diagonal), T (c x b) and h (c)
// are scratch.
thanos_status row_outliers(hipStream_t s, const float* W, const float* H, int64_t c, int64_t b,
                           long long n_out, float* Hf, float* T, float* h, uint8_t* skip) {
  hipLaunchKernelGGL(k_lower_half_diag, dim3((unsigned)ceil_div(b, 256), (unsigned)b), dim3(256), 0,
                     s, H, b, Hf);
  THANOS_LAUNCH_CHECK();
  thanos_status st = gemm_f32(s, false, true, c, b, b, 1.f, W, b, Hf, b, 0.f, T, b, false, true);
  if (st != THANOS_OK) return st;
  hipLaunchKernelGGL(k_rowdot, dim3((unsigned)ceil_div(c, 4)), dim3(256), 0, s, T, W, c, b, h);
  THANOS_LAUNCH_CHECK();
  hipLaunchKernelGGL(k_row_rank, dim3((unsigned)ceil_div(c, 256)), dim3(256), 0, s, h, c,
                     (int64_t)n_out, skip);
  THANOS_LAUNCH_CHECK();
  return THANOS_OK;
}

// ------------------------------------------------------------------------------------------
struct SweepWs {
  float* sx;
  float* Lam;
  float* P;
  unsigned int* hist;
  SelState* st;
  int* row_cand;
  int* row_eq;
  unsigned int* below_part;  // one count per workgroup of the block update
  unsigned int* cand_n;      // per update workgroup: keys inside the selection window ...
  uint2* cand;               // ... and (key, row) of each, kCandStage slots per workgroup
  unsigned long long* binlist;  // k_select: the keys of the threshold's bin
  unsigned int* wgflag;      // k_select: one word per workgroup, a cache line each
  float* Hf;        // alpha > 0: symmetric copy of H, b x b
  float* T;         // alpha > 0: W * H, c x b
  float* h;         // alpha > 0: row losses, c
  uint8_t* row_skip;  // alpha > 0: c
  float* tile_scratch;  // large blocks: tile grids of the rows in flight
  float* Kc;            // inverse of every block's G (B x B per block), or nullptr
};

static char* carve(char*& p, size_t bytes) {
  char* q = p;
  p += align_up(bytes, 256);
  return q;
}

// Blocks whose selection only looks at their own columns (n:m, forced masks) are swept in
// super-blocks of kSuper blocks: inside a super-block the update of a block only reaches the
// end of the super-block, and everything right of it gets one update per super-block with a
// kSuper times longer reduction (the multipliers of all its blocks are kept, c x kSuper*B).
constexpr int kSuper = 8;

// Large blocks (more than 256 unknowns per row, or more than 512 columns): workgroups of
// k_solve_tiled<.., BIG> that run at once, each with a slot for the tile grid of its row.
constexpr int kBigSlots = 512;
static inline bool needs_big(int B, int smax) { return smax > kTlSmax || B > kTlBw; }
static inline int64_t big_slot_floats(int smax) {
  return (int64_t)tl_ntiles((std::min(smax, kBigSmax) + 31) / 32) * kTlSz;
}

static void launch_update(hipStream_t s, UpdateArgs ua, dim3 tiles) {
  ua.gx = (int)tiles.x;
  ua.gy = (int)tiles.y;
  const unsigned rp = (tiles.y + 7) / 8;
  const unsigned n = tiles.y >= 16 ? 8 * rp * tiles.x : tiles.x * tiles.y;
  hipLaunchKernelGGL(k_update, dim3(n), dim3(kXThreads), kUpdSmemBytes, s, ua);
}

// Whether rows that lose more than half of a block are solved through K = G^{-1} (see
// k_comp_blocks, k_solve_tiled): only the tiled solver does it (blocks wider than 128 columns),
// the blocks' K come from the factor of the same call (not available with a given factor), the
// matrix-vector products read K in aligned groups of four columns, and n:m patterns that remove
// at most half of every group never need it.
bool sweep_uses_complement(const thanos_prune_opts* o, int64_t b) {
  const int B = o->block_size;
  if (o->factor_in) return false;
  if (o->mode == THANOS_NM && !o->mask_in && 2 * o->n <= o->m) return false;
  // blocks of up to 128 columns: the one-wavefront solver holds 96 unknowns and takes the rare
  // rows with more through the complement (no alignment needed there); nothing to do when no
  // row can have more
  if (B <= 128) return B > 96 && (o->mode != THANOS_NM || o->mask_in);
  return B % 4 == 0 && b % 4 == 0;
}

size_t sweep_workspace_bytes(int64_t c, int64_t b, int B, bool outliers, int smax, bool comp) {
  size_t n = 0;
  if (comp) n += align_up((size_t)ceil_div(b, B) * B * B * 4, 256);  // K blocks
  if (needs_big(B, smax))
    n += align_up((size_t)std::min<int64_t>(c, kBigSlots) * big_slot_floats(smax) * 4, 256);
  n += align_up((size_t)b * 4, 256);            // sx
  n += align_up((size_t)c * B * kSuper * 4 * 2, 256);  // Lam, two super-block buffers
  n += align_up((size_t)b * b * 4, 256);        // P
  n += align_up(4 * 2048 * 4, 256);             // hist: window + three passes
  n += align_up(sizeof(SelState), 256);         // state
  n += 2 * align_up((size_t)c * 4, 256);        // row_cand, row_eq
  n += align_up((size_t)ceil_div(b, kTN) * ceil_div(c, kTM) * 4, 256);  // below_part
  n += align_up((size_t)ceil_div(b, kTN) * ceil_div(c, kTM) * 4, 256);  // cand_n
  n += align_up((size_t)ceil_div(b, kTN) * ceil_div(c, kTM) * kCandStage * sizeof(uint2), 256);  // cand
  n += align_up((size_t)kBinCap * 8, 256);                              // binlist
  n += align_up((size_t)kSelMaxWgs * kFlagStride * 4, 256);                     // wgflag
  if (outliers) {
    n += align_up((size_t)b * b * 4, 256);      // Hf
    n += align_up((size_t)c * b * 4, 256);      // T
    n += align_up((size_t)c * 4, 256);          // h
    n += align_up((size_t)c, 256);              // row_skip
  }
  return n;
}

static SweepWs carve_ws(void* ws, int64_t c, int64_t b, int B, bool outliers, int smax,
                        bool comp) {
  char* p = reinterpret_cast<char*>(ws);
  SweepWs w;
  w.Kc = nullptr;
  if (comp) w.Kc = reinterpret_cast<float*>(carve(p, (size_t)ceil_div(b, B) * B * B * 4));
  w.tile_scratch = nullptr;
  if (needs_big(B, smax))
    w.tile_scratch = reinterpret_cast<float*>(
        carve(p, (size_t)std::min<int64_t>(c, kBigSlots) * big_slot_floats(smax) * 4));
  w.sx = reinterpret_cast<float*>(carve(p, (size_t)b * 4));
  w.Lam = reinterpret_cast<float*>(carve(p, (size_t)c * B * kSuper * 4 * 2));
  w.P = reinterpret_cast<float*>(carve(p, (size_t)b * b * 4));
  w.hist = reinterpret_cast<unsigned int*>(carve(p, 4 * 2048 * 4));  // window + three passes
  w.st = reinterpret_cast<SelState*>(carve(p, sizeof(SelState)));
  w.row_cand = reinterpret_cast<int*>(carve(p, (size_t)c * 4));
  w.row_eq = reinterpret_cast<int*>(carve(p, (size_t)c * 4));
  w.below_part = reinterpret_cast<unsigned int*>(
      carve(p, (size_t)ceil_div(b, kTN) * ceil_div(c, kTM) * 4));
  w.cand_n = reinterpret_cast<unsigned int*>(
      carve(p, (size_t)ceil_div(b, kTN) * ceil_div(c, kTM) * 4));
  w.cand = reinterpret_cast<uint2*>(
      carve(p, (size_t)ceil_div(b, kTN) * ceil_div(c, kTM) * kCandStage * sizeof(uint2)));
  w.binlist = reinterpret_cast<unsigned long long*>(carve(p, (size_t)kBinCap * 8));
  w.wgflag = reinterpret_cast<unsigned int*>(carve(p, (size_t)kSelMaxWgs * kFlagStride * 4));
  w.Hf = w.T = w.h = nullptr;
  w.row_skip = nullptr;
  if (outliers) {
    w.Hf = reinterpret_cast<float*>(carve(p, (size_t)b * b * 4));
    w.T = reinterpret_cast<float*>(carve(p, (size_t)c * b * 4));
    w.h = reinterpret_cast<float*>(carve(p, (size_t)c * 4));
    w.row_skip = reinterpret_cast<uint8_t*>(carve(p, (size_t)c));
  }
  return w;
}

// Compute units of the current device (k_select launches at most one workgroup per unit).
static int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
    return 32;
  return n;
}

__global__ void k_init_state(SelState* st, long long r) {
  st->r_rem = r;
  st->need_eq = 0;
  st->ties_all = 0;
  st->deferred = 0;
  st->tau = 0u;
  st->none = (r <= 0) ? 1 : 0;
  st->win_lo = 0u;
  st->win_shift = kWinShiftMin;
  st->pred_try = 0;
  st->cand_overflow = 0;
  st->arrived = st->nbin = st->bar = 0u;
}

template <int SEL>
static void launch_solve(hipStream_t s, SolveArgs a, int smax) {
  // tiled solver: rows that lose more than half of the block are solved through the complement
  if (a.Kc && a.bw > 128) smax = SEL == SEL_NM ? std::min(smax, a.bw - smax) : a.bw / 2;
  if (a.bw <= 128 && smax <= 64) {
    constexpr int kWpb = 4;
    const size_t smem = kWpb * sizeof(SolveMfmaSmem<2>);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_solve_mfma<SEL, kWpb, 2>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (SEL == SEL_NM && a.bw * a.n == 64 * a.m && a.bw % a.m == 0) {  // 64 unknowns in every row
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_solve_mfma<SEL, kWpb, 2, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      hipLaunchKernelGGL((k_solve_mfma<SEL, kWpb, 2, true>), dim3((unsigned)ceil_div(a.c, kWpb)),
                         dim3(64 * kWpb), smem, s, a);
      return;
    }
    hipLaunchKernelGGL((k_solve_mfma<SEL, kWpb, 2>), dim3((unsigned)ceil_div(a.c, kWpb)),
                       dim3(64 * kWpb), smem, s, a);
  } else if (a.bw <= 128) {
    // Up to 96 unknowns: one wavefront per row on the matrix cores.  When s varies from row to
    // row (and may exceed 96) the few larger rows get a launch of the 128-thread kernel.
    constexpr int kWpb = 2;
    const size_t smem = kWpb * sizeof(SolveMfmaSmem<3>);
    const bool varies = SEL != SEL_NM;
    if (varies || smax <= 96) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_solve_mfma<SEL, kWpb, 3>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      a.defer_large = (varies && a.bw > 96) ? 1 : 0;
      hipLaunchKernelGGL((k_solve_mfma<SEL, kWpb, 3>), dim3((unsigned)ceil_div(a.c, kWpb)),
                         dim3(64 * kWpb), smem, s, a);
      a.defer_large = 0;
      // rows with more than 96 unknowns: solved by that launch through the complement when the
      // blocks' K are at hand, else by the 128-thread kernel
      if (!(varies && a.bw > 96) || a.Kc) return;
      a.s_min = 97;
    }
    hipLaunchKernelGGL((k_solve_wide<SEL, 128>), dim3((unsigned)a.c), dim3(128), 0, s, a);
  } else if (smax > kTlSmax || a.bw > kTlBw) {
    // large blocks: tile grids in global memory, persistent workgroups (two per compute unit)
    constexpr int kNw = 8;
    a.nt_lo = 0;
    a.nt_max = kBigSmax / 32;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_solve_tiled<SEL, kNw, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)tl_big_smem_bytes());
    hipLaunchKernelGGL((k_solve_tiled<SEL, kNw, true>),
                       dim3((unsigned)std::min<int64_t>(a.c, kBigSlots)), dim3(64 * kNw),
                       tl_big_smem_bytes(), s, a);
  } else {
    // LDS per row grows with the square of the tile rows; systems of up to 160 unknowns leave
    // room for two workgroups per compute unit, so when s varies from row to row (and may be
    // larger) the small rows get a launch of their own.
    const int nt_all = std::max(3, (std::min(smax, kTlSmax) + 31) / 32);
    constexpr int kNtTwo = 5;
    const bool split = SEL != SEL_NM && nt_all > kNtTwo;
    a.nt_lo = 0;
    a.nt_max = split ? kNtTwo : nt_all;
    if (a.nt_max <= 4) {  // small footprint: three workgroups of four wavefronts per compute unit
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_solve_tiled<SEL, 4>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)tl_smem_bytes(4));
      hipLaunchKernelGGL((k_solve_tiled<SEL, 4>), dim3((unsigned)a.c), dim3(256),
                         tl_smem_bytes(a.nt_max), s, a);
      return;
    }
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(k_solve_tiled<SEL, 8>),
                              hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)tl_smem_bytes(kTlSmax / 32));
    hipLaunchKernelGGL((k_solve_tiled<SEL, 8>), dim3((unsigned)a.c), dim3(512),
                       tl_smem_bytes(a.nt_max), s, a);
    if (split) {
      a.nt_lo = kNtTwo + 1;
      a.nt_max = kTlSmax / 32;  // the launch that reports systems beyond the solver's limit
      hipLaunchKernelGGL((k_solve_tiled<SEL, 8>), dim3((unsigned)a.c), dim3(512),
                         tl_smem_bytes(a.nt_max), s, a);
    }
  }
}

// The part of the sweep that needs neither the factor nor the diagonal of H: the fp32 working
// copy of the weights and, with outlier rows, the rows to leave alone.  The caller may run it on
// another stream while the factorisation is going (the two touch disjoint memory) and then
// passes prepared = true to sweep().
thanos_status sweep_prepare(hipStream_t s, const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                            const float* H, const thanos_prune_opts* o, long long n_out, float* W,
                            void* ws) {
  const int B = o->block_size;
  const bool outliers = n_out > 0;
  const int smax_all = (o->mode == THANOS_NM && !o->mask_in) ? B / o->m * o->n : B;
  SweepWs w = carve_ws(ws, c, b, B, outliers, smax_all, sweep_uses_complement(o, b));
  const int64_t n = c * b;
  const unsigned nblk = (unsigned)ceil_div(n, 256);
  if (wdt == THANOS_F32)
    hipLaunchKernelGGL(k_to_f32<float>, dim3(nblk), dim3(256), 0, s, (const float*)W_in, W, n);
  else if (wdt == THANOS_F16)
    hipLaunchKernelGGL(k_to_f32<__half>, dim3(nblk), dim3(256), 0, s, (const __half*)W_in, W, n);
  else
    hipLaunchKernelGGL(k_to_f32<__hip_bfloat16>, dim3(nblk), dim3(256), 0, s,
                       (const __hip_bfloat16*)W_in, W, n);
  THANOS_LAUNCH_CHECK();
  if (outliers) {
    thanos_status st = row_outliers(s, W, H, c, b, n_out, w.Hf, w.T, w.h, w.row_skip);
    if (st != THANOS_OK) return st;
  }
  return THANOS_OK;
}

thanos_status sweep(hipStream_t s, const void* W_in, thanos_dtype wdt, int64_t c, int64_t b,
                    const float* H, const float* U, const float* xnorm2,
                    const thanos_prune_opts* o, long long r_total, long long n_out, float* W,
                    void* W_cast, uint8_t* mask, void* ws, int32_t* info, bool single_stream,
                    PhaseTimer* pt, const float* Lfac, int64_t ldL, bool prepared) {
  const int B = o->block_size;
  const bool outliers = n_out > 0;
  const int smax_all = (o->mode == THANOS_NM && !o->mask_in) ? B / o->m * o->n : B;
  const bool comp = sweep_uses_complement(o, b) && Lfac != nullptr;
  SweepWs w = carve_ws(ws, c, b, B, outliers, smax_all, sweep_uses_complement(o, b));
  const int64_t n = c * b;
  const unsigned nblk = (unsigned)ceil_div(n, 256);

  if (!prepared) {
    thanos_status st = sweep_prepare(s, W_in, wdt, c, b, H, o, n_out, W, ws);
    if (st != THANOS_OK) return st;
  }
  hipLaunchKernelGGL(k_sqrt, dim3((unsigned)ceil_div(b, 256)), dim3(256), 0, s, xnorm2, w.sx, b);
  THANOS_LAUNCH_CHECK();

  const bool aligned_b = (b % 4 == 0) && (B % 4 == 0);
  const int pair_w = (aligned_b && reinterpret_cast<uintptr_t>(W) % 8 == 0 &&
                      reinterpret_cast<uintptr_t>(mask) % 2 == 0) ? 1 : 0;
  {
    BlockRowsArgs a{U, w.P, b, B,
                    (aligned_b && reinterpret_cast<uintptr_t>(U) % 16 == 0) ? 1 : 0};
    dim3 grid((unsigned)ceil_div(b, kTN), (unsigned)ceil_div(b, B), (unsigned)ceil_div(B, kTM));
    THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_block_rows),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)kXSmemBytes));
    THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_update),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         (int)kUpdSmemBytes));
    hipLaunchKernelGGL(k_block_rows, grid, dim3(kXThreads), kXSmemBytes, s, a);
    THANOS_LAUNCH_CHECK();
    if (comp) {
      const unsigned nt32 = (unsigned)ceil_div(B, 32);
      hipLaunchKernelGGL(k_comp_blocks, dim3(nt32, nt32, (unsigned)ceil_div(b, B)), dim3(256), 0, s,
                         Lfac, ldL, b, B, w.Kc);
      THANOS_LAUNCH_CHECK();
    }
  }

  const bool unstructured = (o->mode == THANOS_UNSTRUCTURED) && o->mask_in == nullptr;
  if (unstructured) {
    hipLaunchKernelGGL(k_fill_u32, dim3(32), dim3(256), 0, s, w.hist, (int64_t)4 * 2048, 0u);
    hipLaunchKernelGGL(k_fill_u32, dim3(kSelMaxWgs * kFlagStride / 256), dim3(256), 0, s, w.wgflag,
                       (int64_t)kSelMaxWgs * kFlagStride, 0u);
    hipLaunchKernelGGL(k_init_state, dim3(1), dim3(1), 0, s, w.st, r_total);
    THANOS_LAUNCH_CHECK();
  }

  const unsigned rows4 = (unsigned)ceil_div(c, 4);
  const int super = unstructured ? 1 : kSuper;   // the global residual mask needs current weights
  const int ldl = B * super;
  // The update that reaches right of a super-block is split like the wide update of the
  // factorisation: the columns of the next super-block on the caller's stream, the rest on a
  // second stream next to the (latency-bound) blocks of the next super-block.  The multipliers
  // of consecutive super-blocks alternate between two buffers.
  const int n_super = (int)ceil_div(b, (int64_t)B * super);
  AuxStream aux(s, super > 1 ? 2 * n_super : 0, single_stream);
  if (!aux.ok) return THANOS_ERR_HIP;
  int pending_join = -1;
  int win_parts = 0;  // workgroups of the previous block's update (partial counts to sum)
  for (int64_t j1 = 0; j1 < b; j1 += B) {
    const int bw = (int)std::min<int64_t>(B, b - j1);
    const int64_t blk = j1 / B;
    const int64_t sbi = blk / super;
    const int64_t sb_start = sbi * super * (int64_t)B;
    const int64_t sb_end = (super == 1) ? b : std::min<int64_t>(b, sb_start + (int64_t)super * B);
    const int64_t loff = (super == 1) ? 0 : (j1 - sb_start);
    float* lam_sb = w.Lam + (sbi & 1) * (int64_t)c * ldl;
    if (unstructured) {
      phase_mark(pt, THANOS_PHASE_MASK);
      // 16-byte loads need W + i*b + j1 and sx + j1 aligned (W, sx come 256-byte aligned)
      const int sel_vec = (b % 4 == 0 && j1 % 4 == 0 &&
                           reinterpret_cast<uintptr_t>(W) % 16 == 0) ? 1 : 0;
      // the previous block's update counted the window around its threshold, and listed the
      // keys inside it, while it wrote the new weights
      SelectArgs ga;
      ga.W = W;
      ga.sx = w.sx;
      ga.st = w.st;
      ga.hist = w.hist;
      ga.below_part = w.below_part;
      ga.n_part = win_parts;
      ga.cand_n = w.cand_n;
      ga.cand = w.cand;
      ga.binlist = w.binlist;
      ga.row_cnt = w.row_cand;
      ga.row_cand = w.row_cand;
      ga.row_eq = w.row_eq;
      ga.tau_out = o->threshold_out ? o->threshold_out + blk : nullptr;
      ga.info = info;
      ga.c = c;
      ga.b = b;
      ga.j1 = j1;
      ga.first = j1 == 0 ? 1 : 0;
      ga.vec = sel_vec;
      ga.seq = (unsigned int)(blk + 1);
      ga.wgflag = w.wgflag;
      const unsigned sel_wgs = (unsigned)std::min<int64_t>(std::min(kSelMaxWgs, compute_units()),
                                                           ceil_div(c, kSelThreads / 64));
      hipLaunchKernelGGL(k_select, dim3(sel_wgs), dim3(kSelThreads), 0, s, ga);
      THANOS_LAUNCH_CHECK();
    }
    phase_mark(pt, THANOS_PHASE_SOLVE);
    SolveArgs sa;
    sa.W = W;
    sa.P = w.P;
    sa.sx = w.sx;
    sa.mask_in = o->mask_in;
    sa.mask_out = mask;
    sa.Lam = lam_sb + loff;
    sa.st = w.st;
    sa.st_rw = w.st;
    sa.row_skip = w.row_skip;
    sa.row_eq = w.row_eq;
    sa.row_cnt = w.row_cand;  // free once k_select has read the candidate flags
    sa.info = info;
    sa.c = c;
    sa.b = b;
    sa.j1 = j1;
    sa.bw = bw;
    sa.ldl = ldl;
    sa.n = o->n;
    sa.m = o->m;
    sa.nt_lo = sa.nt_max = 0;
    sa.s_min = 0;
    sa.defer_large = 0;
    sa.tile_scratch = w.tile_scratch;
    sa.slot_floats = big_slot_floats(smax_all);
    sa.Kc = comp ? w.Kc + blk * (int64_t)B * B : nullptr;
    sa.ldk = B;
    if (o->mask_in) {
      launch_solve<SEL_GIVEN>(s, sa, bw);
    } else if (o->mode == THANOS_NM) {
      launch_solve<SEL_NM>(s, sa, bw / o->m * o->n);
    } else {
      launch_solve<SEL_THRESHOLD>(s, sa, bw);
    }
    THANOS_LAUNCH_CHECK();

    phase_mark(pt, THANOS_PHASE_UPDATE);
    {  // this block's update, up to the end of its super-block
      dim3 grid((unsigned)ceil_div(sb_end - j1, kTN), (unsigned)ceil_div(c, kTM));
      const bool feed = unstructured && j1 + bw < b;  // a next block exists: count its window
      if (feed) win_parts = (int)(grid.x * grid.y);
      UpdateArgs ua{W, lam_sb + loff, w.P, mask, c, b, j1, j1, sb_end, j1, j1 + bw, bw, ldl,
                    (B % 4 == 0) ? 1 : 0, aligned_b ? 1 : 0, pair_w,
                    feed ? w.hist : nullptr, w.below_part, w.cand_n, w.cand, w.st, w.sx};
      launch_update(s, ua, grid);
      THANOS_LAUNCH_CHECK();
    }
    if (super > 1 && j1 + bw == sb_end && sb_end < b) {  // all blocks of the super-block
      const int64_t next_end = std::min<int64_t>(b, sb_end + (int64_t)super * B);
      const int kk = (int)(sb_end - sb_start);
      // The strip (the columns of the next super-block) first: the next block's solve waits for
      // it, so it gets the chip before the much larger rest does.  It was last written by the
      // previous rest.
      if (pending_join >= 0) THANOS_CHECK(aux.join(pending_join));
      {
        UpdateArgs ua{W, lam_sb, w.P, mask, c, b, sb_start, sb_end, next_end, 0, 0, kk, ldl,
                      (B % 4 == 0) ? 1 : 0, aligned_b ? 1 : 0, pair_w, nullptr, nullptr, nullptr, nullptr,
                      nullptr, nullptr};
        dim3 grid((unsigned)ceil_div(next_end - sb_end, kTN), (unsigned)ceil_div(c, kTM));
        launch_update(s, ua, grid);
        THANOS_LAUNCH_CHECK();
      }
      if (next_end < b) {  // rest: right of the next super-block, second stream
        THANOS_CHECK(aux.fork((int)(2 * sbi)));
        UpdateArgs ua{W, lam_sb, w.P, mask, c, b, sb_start, next_end, b, 0, 0, kk, ldl,
                      (B % 4 == 0) ? 1 : 0, aligned_b ? 1 : 0, pair_w, nullptr, nullptr, nullptr, nullptr,
                      nullptr, nullptr};
        dim3 grid((unsigned)ceil_div(b - next_end, kTN), (unsigned)ceil_div(c, kTM));
        launch_update(aux.stream, ua, grid);
        THANOS_LAUNCH_CHECK();
        THANOS_CHECK(aux.record((int)(2 * sbi + 1)));
        pending_join = (int)(2 * sbi + 1);
      }
    }
  }
  if (pending_join >= 0) THANOS_CHECK(aux.join(pending_join));

  phase_mark(pt, THANOS_PHASE_FINALISE);
  if (W_cast) {
    if (wdt == THANOS_F32)
      hipLaunchKernelGGL(k_from_f32<float>, dim3(nblk), dim3(256), 0, s, W, (float*)W_cast, n);
    else if (wdt == THANOS_F16)
      hipLaunchKernelGGL(k_from_f32<__half>, dim3(nblk), dim3(256), 0, s, W, (__half*)W_cast, n);
    else
      hipLaunchKernelGGL(k_from_f32<__hip_bfloat16>, dim3(nblk), dim3(256), 0, s, W,
                         (__hip_bfloat16*)W_cast, n);
    THANOS_LAUNCH_CHECK();
  }
  return THANOS_OK;
}

}  // namespace thanos

#ifdef THANOS_TIMELINE
// Diagnostic build only (see timeline.h): which launch to record, and the recorded timestamps.
extern "C" int thanos_timeline_select(int grid_workgroups) {
  return (int)hipMemcpyToSymbol(HIP_SYMBOL(thanos::g_timeline_grid), &grid_workgroups, sizeof(int));
}
extern "C" int thanos_timeline_read(unsigned long long* host, size_t bytes) {
  if (bytes > sizeof(unsigned long long) * thanos::kTlWgs * thanos::kTlSlots) return -1;
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(thanos::g_timeline), bytes);
}
extern "C" int thanos_timeline_clear(void) {
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(thanos::g_timeline)) != hipSuccess) return -1;
  return (int)hipMemset(p, 0, sizeof(unsigned long long) * thanos::kTlWgs * thanos::kTlSlots);
}
#endif

