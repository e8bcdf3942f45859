// 128x128 fp32 tile product on the CDNA4 bf16 matrix cores with three-way operand splitting.
//
// An fp32 value x is written as x = x1 + x2 + x3 with x1 = bf16(x), x2 = bf16(x - x1),
// x3 = bf16(x - x1 - x2): 3 x 8 significant bits, the remainders are exact in fp32.  The product
// a*b is then the sum of the six partial products whose weight is at least 2^-16 relative,
//     a1 b1 + (a1 b2 + a2 b1) + (a1 b3 + a2 b2 + a3 b1),
// each exact in the fp32 accumulator of v_mfma_f32_32x32x16_bf16; what is dropped is of order
// 2^-24 |a||b|, the size of one fp32 rounding.  Six bf16 MFMAs of 32 cycles replace eight fp32
// MFMAs (32x32x2) of 64 cycles for the same 32x32x16 block of products, and draw less power.
//
// One workgroup of 512 threads = 8 wavefronts with different jobs (a wavefront cannot overlap
// its own vector arithmetic with its own MFMAs, two wavefronts of a SIMD can):
//   wavefronts 0..3 (consumers): 2x2 arrangement, each owns 64x64 = 2x2 MFMA tiles of the
//       accumulator (same layout as gemm_tile.h); per slab of 32 k-values they read their
//       operands from LDS (16 bytes per lane and fragment) and issue 48 MFMAs;
//   wavefronts 4..7 (producers): 4,5 fetch the A slab, 6,7 the B slab (32 floats per thread),
//       split them in registers and store three bf16 planes per operand in LDS as
//       [row][32 k] (row stride 80 bytes: the 16-byte reads of consecutive rows then cover all
//       banks).  The global loads of the next slab are issued right after the stores.
// One LDS buffer of 60 KB and two barriers per slab (filled / consumed): inside a workgroup
// filling and multiplying alternate, and the overlap comes from the SECOND workgroup that the
// small footprint (<= 128 registers, 68 KB of LDS with the staged write-out) lets a compute unit
// hold.  Two buffers in one workgroup per unit (122 KB) were 15 % slower on large products:
// every barrier stalled the whole unit.  After the call only wavefronts 0..3 hold the result.
#pragma once
#include "gemm_tile.h"
#include "timeline.h"

namespace thanos {

constexpr int kXK = 32;                      // k-values per slab
constexpr int kXRow = 80;                    // bytes per LDS row: 32 bf16 + 16 bytes of padding
constexpr int kXPlane = 128 * kXRow;         // one bf16 plane of one operand
constexpr int kXThreads = 512;
// LDS of a workgroup: the six operand planes of one slab (61 440 bytes), reused for the staged
// output tile (128 rows of 544 bytes), whichever is larger
constexpr size_t kXSmemBytes = (6 * (size_t)kXPlane > 128 * 544) ? 6 * (size_t)kXPlane : 128 * 544;

// LDS view: {a, b} x plane[3] (buf is always 0: one buffer)
__device__ __forceinline__ char* x3_plane(char* smem, int buf, int operand, int plane) {
  return smem + ((buf * 2 + operand) * 3 + plane) * kXPlane;
}

// 32 floats of one operand slab held by a producer thread.
//   !KMAJOR: v[q] = row m = (u >> 3) + 16 q, k = 4*(u & 7) .. +3.
//    KMAJOR: v[q] = the four rows m = 4*(u & 31) .. +3 at k = 8*(u >> 5) + q.
struct SlabRegsX3 {
  float4 v[8];
  uint32_t ok;  // fast path: bit q set = piece q is inside the operand (else v[q] is junk)
};

// Per-thread source of an operand: pointers to its eight 16-byte pieces of the slab at
// k = kbeg, the step from one slab to the next, and how much of each piece exists.
struct SlabSrcX3 {
  const float* p[8];
  int64_t step;  // floats between consecutive slabs
  int kofs[8];   // k offset of piece q inside the slab
  int nrow;      // KMAJOR: number of valid rows (0..4) of every piece
  bool row_ok[8];
};

template <bool KMAJOR>
__device__ __forceinline__ void slab_src_x3(SlabSrcX3& s, const float* __restrict__ P, int64_t ld,
                                            int ext, int kbeg, int u) {
  s.nrow = 4;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    if (KMAJOR) {
      const int m4 = 4 * (u & 31);
      s.kofs[q] = 8 * (u >> 5) + q;
      s.p[q] = P + (int64_t)(kbeg + s.kofs[q]) * ld + m4;
      s.nrow = min(4, max(0, ext - m4));
      s.row_ok[q] = m4 < ext;
    } else {
      const int m = (u >> 3) + 16 * q;
      s.kofs[q] = 4 * (u & 7);
      s.p[q] = P + (int64_t)m * ld + kbeg + s.kofs[q];
      s.row_ok[q] = m < ext;
    }
  }
  s.step = KMAJOR ? (int64_t)kXK * ld : (int64_t)kXK;
}

// Loads slab number `it` (k0 = kbeg + it*kXK); krem = kend - k0 (<= 0: nothing is read).
// FAST: every piece is either completely inside the operand or completely outside (the caller
// checked alignment and that the extents are multiples of 4).  The loads are then issued
// unconditionally (from a safe address when outside) and outside pieces are zeroed when the
// slab is split: straight-line code with no early use of the data, so that the compiler can
// keep the newer of the two slabs in flight while it waits for the older one.  Conditional
// loads, or a select right behind the load, force it to wait for all of them.
template <bool KMAJOR, bool FAST>
__device__ __forceinline__ void slab_load_x3(SlabRegsX3& r, const SlabSrcX3& s, int it, int krem,
                                             const float* __restrict__ safe) {
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const float* p = s.p[q] + (int64_t)it * s.step;
    if (FAST) {
      // no use of the loaded value here: the zeroing of outside pieces happens when the slab
      // is split, so that nothing waits for these loads before then
      const bool ok = s.row_ok[q] && s.kofs[q] < krem;
      r.v[q] = *reinterpret_cast<const float4*>(ok ? p : safe);
      if (q == 0) r.ok = 0;
      r.ok |= ok ? (1u << q) : 0u;
      continue;
    }
    float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
    if (KMAJOR) {
      if (s.kofs[q] < krem && s.row_ok[q]) {
        val.x = p[0];
        if (s.nrow > 1) val.y = p[1];
        if (s.nrow > 2) val.z = p[2];
        if (s.nrow > 3) val.w = p[3];
      }
    } else {
      const int kr = krem - s.kofs[q];  // valid k-values from this piece on
      if (s.row_ok[q] && kr > 0) {
        val.x = p[0];
        if (kr > 1) val.y = p[1];
        if (kr > 2) val.z = p[2];
        if (kr > 3) val.w = p[3];
      }
    }
    r.v[q] = val;
  }
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Split two floats into three packed bf16 pairs (conversion = the packed two-at-a-time
// instruction, the way back is a shift / a mask).
__device__ __forceinline__ void split2(float x0, float x1, uint32_t (&packed)[3]) {
  f32x2 v = {x0, x1};
#pragma unroll
  for (int p = 0; p < 3; ++p) {
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    packed[p] = __builtin_bit_cast(uint32_t, h);
    if (p < 2) {
      v[0] -= __uint_as_float(packed[p] << 16);
      v[1] -= __uint_as_float(packed[p] & 0xffff0000u);
    }
  }
}

template <bool KMAJOR, bool MASKED>
__device__ __forceinline__ void slab_store_x3(char* smem, int buf, int operand,
                                              const SlabRegsX3& rin, int u) {
  SlabRegsX3 r = rin;
  if (MASKED) {
#pragma unroll
    for (int q = 0; q < 8; ++q)
      if (!((r.ok >> q) & 1)) r.v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  char* pl[3] = {x3_plane(smem, buf, operand, 0), x3_plane(smem, buf, operand, 1),
                 x3_plane(smem, buf, operand, 2)};
  if (KMAJOR) {
    // row m4 + mm: the 8 k-values 8*(u>>5) .. +7 -> 16 bytes per plane
    const int m4 = 4 * (u & 31), kb = 16 * (u >> 5);
#pragma unroll
    for (int mm = 0; mm < 4; ++mm) {
      float c[8];
#pragma unroll
      for (int q = 0; q < 8; ++q)
        c[q] = mm == 0 ? r.v[q].x : mm == 1 ? r.v[q].y : mm == 2 ? r.v[q].z : r.v[q].w;
      u32x4 o[3];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        uint32_t pk[3];
        split2(c[2 * e], c[2 * e + 1], pk);
        o[0][e] = pk[0];
        o[1][e] = pk[1];
        o[2][e] = pk[2];
      }
#pragma unroll
      for (int p = 0; p < 3; ++p)
        *reinterpret_cast<u32x4*>(pl[p] + (m4 + mm) * kXRow + kb) = o[p];
    }
  } else {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      uint32_t lo2[3], hi2[3];
      split2(r.v[q].x, r.v[q].y, lo2);
      split2(r.v[q].z, r.v[q].w, hi2);
      const int off = ((u >> 3) + 16 * q) * kXRow + 8 * (u & 7);
#pragma unroll
      for (int p = 0; p < 3; ++p)
        *reinterpret_cast<uint2*>(pl[p] + off) = make_uint2(lo2[p], hi2[p]);
    }
  }
}

// Producer of a reduction of exactly four whole slabs (K = 128: the block updates of the sweep,
// panel and narrow updates of the factorisation), whole aligned operand.  Two slabs are in
// flight: the loads of slab it + 2 are requested as soon as the registers of slab it have gone
// to LDS, so a load has two multiply phases to arrive in; with one slab ahead (the loop below)
// the producers wait for memory in every slab, which is a third of so short a product.  Written
// without a loop: across a loop edge the compiler waits for ALL outstanding loads.
template <bool KMAJOR>
__device__ __forceinline__ void x3_produce4(char* smem, int operand, const float* __restrict__ P,
                                            int64_t ld, int ext, int kbeg, int u) {
  SlabSrcX3 src;
  slab_src_x3<KMAJOR>(src, P, ld, ext, kbeg, u);
  SlabRegsX3 r0, r1;
  slab_load_x3<KMAJOR, true>(r0, src, 0, 4 * kXK, P);
  slab_load_x3<KMAJOR, true>(r1, src, 1, 3 * kXK, P);
  slab_store_x3<KMAJOR, false>(smem, 0, operand, r0, u);
  slab_load_x3<KMAJOR, true>(r0, src, 2, 2 * kXK, P);
  __syncthreads();
  __syncthreads();
  slab_store_x3<KMAJOR, false>(smem, 0, operand, r1, u);
  slab_load_x3<KMAJOR, true>(r1, src, 3, kXK, P);
  __syncthreads();
  __syncthreads();
  slab_store_x3<KMAJOR, false>(smem, 0, operand, r0, u);
  __syncthreads();
  __syncthreads();
  slab_store_x3<KMAJOR, false>(smem, 0, operand, r1, u);
  __syncthreads();
  __syncthreads();
}

// Producer loop of one operand: split and store slab `it`, request slab `it + 1`, then the two
// barriers of the slab (the consumers run the same barrier sequence).
template <bool KMAJOR, bool FAST, bool MASKED>
__device__ __forceinline__ void x3_produce(char* smem, int operand, const float* __restrict__ P,
                                           int64_t ld, int ext, int kbeg, int kend, int nslab,
                                           int u) {
  SlabSrcX3 src;
  slab_src_x3<KMAJOR>(src, P, ld, ext, kbeg, u);
  const int klen = kend - kbeg;
  SlabRegsX3 r;
  slab_load_x3<KMAJOR, FAST>(r, src, 0, klen, P);
  for (int it = 0; it < nslab; ++it) {
    if (operand == 0 && u < 64) TL_MARK(8 + 4 * it);
    slab_store_x3<KMAJOR, MASKED>(smem, 0, operand, r, u);
    slab_load_x3<KMAJOR, FAST>(r, src, it + 1, klen - (it + 1) * kXK, P);
    if (operand == 0 && u < 64) TL_MARK(8 + 4 * it + 1);
    __syncthreads();  // slab it is in LDS
    __syncthreads();  // consumers are done with it
  }
}

// acc += op(A)[0:128, kbeg:kend] * op(B)[kbeg:kend, 0:128]; arguments as in gemm_tile(), smem =
// kXSmemBytes of LDS, called by all 512 threads; the result is in wavefronts 0..3.
template <bool A_KMAJOR, bool B_KMAJOR>
__device__ __forceinline__ void gemm_tile_x3(TileAcc& acc, char* smem, const float* __restrict__ A,
                                             int64_t lda, int m_ext, const float* __restrict__ B,
                                             int64_t ldb, int n_ext, int kbeg, int kend, bool vec_a,
                                             bool vec_b) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (kend <= kbeg) return;
  const int nslab = (kend - kbeg + kXK - 1) / kXK;
  __syncthreads();  // previous users of the LDS buffers are done
  if (wave >= 4) {
    // ---------------------------------------------------------------- producers
    // fast path: aligned operand whose extent along the 4-element pieces is a multiple of 4
    const int u = tid & 127;
    // fast: aligned operand whose extent along the 4-element pieces is a multiple of 4;
    // whole: all 128 rows exist and the k range is a whole number of slabs (nothing to zero)
    const bool ktail = (kend - kbeg) % kXK != 0;
    if (wave >= 6) {
      const bool fast = vec_b && (B_KMAJOR ? n_ext % 4 == 0 : (kend - kbeg) % 4 == 0);
      const bool whole = n_ext == 128 && !ktail;
      if (fast && whole && kend - kbeg == 4 * kXK) x3_produce4<B_KMAJOR>(smem, 1, B, ldb, n_ext, kbeg, u);
      else if (fast && whole) x3_produce<B_KMAJOR, true, false>(smem, 1, B, ldb, n_ext, kbeg, kend, nslab, u);
      else if (fast) x3_produce<B_KMAJOR, true, true>(smem, 1, B, ldb, n_ext, kbeg, kend, nslab, u);
      else x3_produce<B_KMAJOR, false, false>(smem, 1, B, ldb, n_ext, kbeg, kend, nslab, u);
    } else {
      const bool fast = vec_a && (A_KMAJOR ? m_ext % 4 == 0 : (kend - kbeg) % 4 == 0);
      const bool whole = m_ext == 128 && !ktail;
      if (fast && whole && kend - kbeg == 4 * kXK) x3_produce4<A_KMAJOR>(smem, 0, A, lda, m_ext, kbeg, u);
      else if (fast && whole) x3_produce<A_KMAJOR, true, false>(smem, 0, A, lda, m_ext, kbeg, kend, nslab, u);
      else if (fast) x3_produce<A_KMAJOR, true, true>(smem, 0, A, lda, m_ext, kbeg, kend, nslab, u);
      else x3_produce<A_KMAJOR, false, false>(smem, 0, A, lda, m_ext, kbeg, kend, nslab, u);
    }
  } else {
    // ---------------------------------------------------------------- consumers
    const int wm = wave >> 1, wn = wave & 1;
    const int lo = lane & 31, hi = lane >> 5;
    const int a_off = (wm * 64 + lo) * kXRow + 16 * hi;
    const int b_off = (wn * 64 + lo) * kXRow + 16 * hi;
    auto compute = [&](int buf) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        bf16x8 af[2][3], bf[2][3];
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
          for (int p = 0; p < 3; ++p) {
            af[f][p] = *reinterpret_cast<const bf16x8*>(x3_plane(smem, buf, 0, p) + a_off +
                                                        f * 32 * kXRow + 32 * ks);
            bf[f][p] = *reinterpret_cast<const bf16x8*>(x3_plane(smem, buf, 1, p) + b_off +
                                                        f * 32 * kXRow + 32 * ks);
          }
        // smallest partial products first; consecutive MFMAs go to different accumulators
        constexpr int pa[6] = {2, 1, 0, 1, 0, 0};
        constexpr int pb[6] = {0, 1, 2, 0, 1, 0};
#pragma unroll
        for (int t = 0; t < 6; ++t)
#pragma unroll
          for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int g = 0; g < 2; ++g)
              acc.v[f][g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[f][pa[t]], bf[g][pb[t]],
                                                                    acc.v[f][g], 0, 0, 0);
      }
    };
    for (int it = 0; it < nslab; ++it) {
      __syncthreads();  // slab it is in LDS
      if (wave == 0) TL_MARK(8 + 4 * it + 2);
      compute(0);
      if (wave == 0) TL_MARK(8 + 4 * it + 3);
      __syncthreads();  // done with it
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Write-out through LDS.  In the accumulator layout a store instruction of a wavefront covers
// two 128-byte pieces of two different rows of C, and only the four multiplying wavefronts hold
// data: 64 loads and 64 stores per thread for a read-modify-write, to rows that lie a whole row
// of the big matrix apart.  Staged in LDS as plain fp32 rows (free once the product is done), the
// tile is walked row by row by all eight wavefronts: a wavefront handles a full 512-byte row per
// instruction, 16 rows each.
constexpr int kXCLd = 136;  // floats per staged row (544 bytes: the two halves of a wavefront, four
                            // rows apart, then write to disjoint banks)
static_assert((size_t)kTM * kXCLd * sizeof(float) <= kXSmemBytes, "staged tile fits the LDS");

// Called by all 512 threads right after gemm_tile_x3 (whose last barrier made the LDS free).
__device__ __forceinline__ const float* x3_stage_tile(const TileAcc& acc, char* smem) {
  float* C = reinterpret_cast<float*>(smem);
  if (threadIdx.x < 256) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int col = acc_col(wn, g, lane);
#pragma unroll
        for (int r = 0; r < 16; ++r) C[acc_row(wm, f, r, lane) * kXCLd + col] = acc.v[f][g][r];
      }
  }
  __syncthreads();
  return C;
}

// Whole, aligned tile: C[0:128, 0:128] = scale * acc (C 8-byte aligned, ldc even).  All 512 threads.
__device__ __forceinline__ void x3_write_tile(const TileAcc& acc, char* smem, float* C,
                                              int64_t ldc, float scale) {
  const float* T = x3_stage_tile(acc, smem);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = wave + 8 * i;
    const float2 t = *reinterpret_cast<const float2*>(T + row * kXCLd + 2 * lane);
    *reinterpret_cast<float2*>(C + (int64_t)row * ldc + 2 * lane) =
        make_float2(scale * t.x, scale * t.y);
  }
}

}  // namespace thanos
