// thanos_hessian_accumulate: H += alpha * Xc^T Xc on the CDNA4 matrix cores.
//
// Xc is token-major [n_tok, b] (16-bit floats), so both MFMA operands of H = Xc^T Xc are
// "channel-contiguous": the reduction index (token) is the strided one, while the 16-bit MFMA
// wants 8 consecutive reduction values per lane.
//
// Workgroup = 256 threads = 4 wavefronts (2x2), tile = 256 x 256 outputs, each wavefront
// 128 x 128 = 4x4 MFMA 32x32x16 tiles (256 accumulator registers).  Only tiles on or below the
// diagonal are computed.  Workgroups are renumbered so that the 32 workgroups resident on one
// XCD work on a 4 x 8 patch of neighbouring tiles and share their panels of X through that
// XCD's L2.
//
// Main kernel (k_syrk16_dma; 16-byte aligned rows, b % 8 == 0):
//   * global -> LDS without registers: buffer_load_dwordx4 ... lds.  One wavefront-wide load
//     moves one token row of both panels (2 x 256 channels = 1 KB) into one LDS row; rows past
//     n_tok are outside the buffer descriptor and arrive as zeros.  Four stages of 32 tokens
//     (row stride 1088 B) keep three k-steps (96 KB per workgroup) in flight.
//   * LDS -> MFMA operand with the transposing read ds_read_b64_tr_b16: within 16 lanes, lane
//     s fetches 8 bytes of row (s / 4), channels 4 (s % 4)..+3, and receives the four rows of
//     ONE channel, i.e. four consecutive reduction values; two such reads make an operand.
//     The 64-byte row padding spreads the four rows of a read over all 64 banks.
//   * one barrier per k-step: wait for the own loads of the next step (vmcnt), barrier, then
//     multiply with the operand reads of the following slice and the loads four steps ahead
//     (into the stage that was consumed last) interleaved one by one between the MFMAs.
// Fallback kernel (k_syrk16; any alignment, any b): 8x8 patches are loaded with guarded scalar
// loads, transposed in registers (v_perm_b32) and written to LDS already k-packed; fragment f
// of a panel is the channel set {8x + f}, which keeps both LDS directions conflict-free.
#include <algorithm>

#include "common.h"
#include "gemm_tile.h"

namespace thanos {

constexpr int kSyTile = 256;  // outputs per tile side
constexpr int kSyKT = 64;     // tokens per k-step
constexpr int kSyOct = kSyKT / 8;

struct SyrkArgs {
  float* H;
  const uint16_t* X;
  int64_t b, n_tok, ldx;
  float alpha;
  int nt;      // tiles per side
  int ntiles;  // nt*(nt+1)/2
  int nsplit;  // k-chunks per tile (main kernel only); > 1: partial sums are added atomically
};

// Logical tile index -> (ti, tj), ti >= tj.  Tiles are ordered by "super-rows" of 4 tile rows,
// column by column inside a super-row, so that 32 consecutive indices cover about 4 x 8 tiles.
__device__ __forceinline__ void tile_from_index(int id, int nt, int& ti, int& tj) {
  int R = 0;
  for (;;) {
    const int r0 = 4 * R;
    const int r1 = min(r0 + 3, nt - 1);
    const int h = r1 - r0 + 1;
    int cnt = 0;
    for (int a = r0; a <= r1; ++a) cnt += a + 1;
    if (id < cnt) {
      const int full = (r0 + 1) * h;
      if (id < full) {
        tj = id / h;
        ti = r0 + id % h;
      } else {
        id -= full;
        for (int c = r0 + 1; c <= r1; ++c) {
          const int n = r1 - c + 1;
          if (id < n) {
            tj = c;
            ti = c + id;
            return;
          }
          id -= n;
        }
      }
      return;
    }
    id -= cnt;
    ++R;
  }
}

template <bool BF16>
__device__ __forceinline__ f32x16 mfma16(const u32x4& a, const u32x4& b, const f32x16& c) {
  if constexpr (BF16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
}

// 8 tokens x 8 channels patch: rows[r] = 8 channels of token r (4 dwords).
struct Patch {
  u32x4 rows[8];
};

template <bool VEC>
__device__ __forceinline__ void patch_load(Patch& p, const uint16_t* __restrict__ X, int64_t ldx,
                                           int64_t tok0, int64_t n_tok, int64_t ch0, int64_t b) {
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    u32x4 v = {0u, 0u, 0u, 0u};
    const int64_t t = tok0 + r;
    if (t < n_tok && ch0 < b) {
      const uint16_t* src = X + t * ldx + ch0;
      if (VEC) {
        v = *reinterpret_cast<const u32x4*>(src);
      } else {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (ch0 + e < b) w[e >> 1] |= (uint32_t)src[e] << (16 * (e & 1));
        v = u32x4{w[0], w[1], w[2], w[3]};
      }
    }
    p.rows[r] = v;
  }
}

// Channel i of the patch as 8 consecutive tokens (4 dwords).
__device__ __forceinline__ u32x4 patch_column(const Patch& p, int i) {
  const int e = i >> 1;
  const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
  u32x4 o;
  o.x = __builtin_amdgcn_perm(p.rows[1][e], p.rows[0][e], sel);
  o.y = __builtin_amdgcn_perm(p.rows[3][e], p.rows[2][e], sel);
  o.z = __builtin_amdgcn_perm(p.rows[5][e], p.rows[4][e], sel);
  o.w = __builtin_amdgcn_perm(p.rows[7][e], p.rows[6][e], sel);
  return o;
}

template <bool BF16, bool VEC>
__global__ __launch_bounds__(256) void k_syrk16(SyrkArgs a) {
  // stage[buf][octet][slot]: slot = side*256 + (channel%8)*32 + channel/8 within the panel
  extern __shared__ u32x4 stage[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int lo = lane & 31, hi = lane >> 5;

  // XCD-aware renumbering: hardware deals workgroups to the 8 XCDs round-robin.
  const int nwg = a.ntiles;
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int logical = xcd * (nwg >> 3) + min(xcd, nwg & 7) + local;
  int ti, tj;
  tile_from_index(logical, a.nt, ti, tj);
  const int64_t i0 = (int64_t)ti * kSyTile, j0 = (int64_t)tj * kSyTile;

  // producer role: this thread moves the patch (octet = wave + 4u, channel group cg)
  const int cg = lane;  // 0..31: i-side panel, 32..63: j-side panel
  const int64_t ch0 = (cg < 32 ? i0 : j0) + 8 * (cg & 31);
  const int slot0 = (cg < 32 ? 0 : 256) + (cg & 31);

  f32x16 acc[4][4];
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[f][g][r] = 0.f;

  const int64_t nkt = (a.n_tok + kSyKT - 1) / kSyKT;
  Patch p[2];
  auto load_tile = [&](int64_t kt) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
      patch_load<VEC>(p[u], a.X, a.ldx, kt * kSyKT + 8 * (wave + 4 * u), a.n_tok, ch0, a.b);
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      u32x4* dst = stage + ((buf * kSyOct + (wave + 4 * u)) * 512 + slot0);
#pragma unroll
      for (int i = 0; i < 8; ++i) dst[i * 32] = patch_column(p[u], i);
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();
  for (int64_t kt = 0; kt < nkt; ++kt) {
    const int buf = (int)(kt & 1);
    if (kt + 1 < nkt) load_tile(kt + 1);
#pragma unroll
    for (int ks = 0; ks < kSyKT / 16; ++ks) {
      const u32x4* base = stage + (buf * kSyOct + 2 * ks + hi) * 512;
      u32x4 af[4], bf[4];
#pragma unroll
      for (int f = 0; f < 4; ++f) af[f] = base[(4 * wm + f) * 32 + lo];
#pragma unroll
      for (int g = 0; g < 4; ++g) bf[g] = base[256 + (4 * wn + g) * 32 + lo];
#pragma unroll
      for (int f = 0; f < 4; ++f)
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[f][g] = mfma16<BF16>(af[f], bf[g], acc[f][g]);
    }
    if (kt + 1 < nkt) store_tile(buf ^ 1);
    __syncthreads();
  }

  // H[i][j] += alpha * acc for i >= j.  MFMA row m <-> channel i0 + 8m + (4wm+f),
  // MFMA column n <-> channel j0 + 8n + (4wn+g).
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int64_t j = j0 + 8 * lo + (4 * wn + g);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = 8 * (r >> 2) + 4 * hi + (r & 3);
        const int64_t i = i0 + 8 * m + (4 * wm + f);
        if (i < a.b && j <= i) {
          float* ptr = a.H + i * a.b + j;
          *ptr += a.alpha * acc[f][g][r];
        }
      }
    }
}

// ------------------------------------------------------------------------------------------
constexpr int kDmaKT = 32;                 // tokens per k-step
constexpr int kDmaStages = 4;
constexpr int kDmaRow = 1024 + 64;         // bytes per LDS token row (2 x 256 channels + pad)
constexpr int kDmaStageBytes = kDmaKT * kDmaRow;

typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 frag_read_tr(const char* lds_lane_base, int byte_off) {
  // two transposing reads: tokens +0..3 and +4..7 of this lane's channel
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds_lane_base + byte_off));
  const s16x4 hi4 =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(lds_lane_base + byte_off + 4 * kDmaRow));
  u32x4 o;
  o.x = (uint16_t)lo4[0] | ((uint32_t)(uint16_t)lo4[1] << 16);
  o.y = (uint16_t)lo4[2] | ((uint32_t)(uint16_t)lo4[3] << 16);
  o.z = (uint16_t)hi4[0] | ((uint32_t)(uint16_t)hi4[1] << 16);
  o.w = (uint16_t)hi4[2] | ((uint32_t)(uint16_t)hi4[3] << 16);
  return o;
}

// One wavefront-wide 16-byte-per-lane load straight into LDS: lane l's 16 bytes land at
// lds_addr + 16*l.  Written as inline assembly so that the compiler's wait-count insertion does
// not serialise every LDS read behind all outstanding loads; the kernel waits explicitly.
__device__ __forceinline__ void dma_row(const u32x4& rsrc, uint32_t lds_addr, uint32_t voff,
                                        uint32_t soff) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "buffer_load_dwordx4 %1, %2, %3 offen lds"
      :
      : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
      : "memory");
}

// NW = 8 wavefronts (two per SIMD): wavefront tile 128 x 64, so that one wavefront of a SIMD
// can fetch operands / wait at the barrier while the other one feeds the matrix core.
// NW = 4: wavefront tile 128 x 128 (fewer LDS reads per MFMA, nothing to overlap with).
template <bool BF16, int NW>
__global__ __launch_bounds__(64 * NW, NW / 4) void k_syrk16_dma(SyrkArgs a) {
  constexpr int WN = NW / 2;          // wavefronts along the column panel
  constexpr int GN = 8 / WN;          // 32-wide MFMA tiles per wavefront along columns
  constexpr int RPW = kDmaKT / NW;    // token rows each wavefront loads per k-step
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int lo = lane & 31, hi = lane >> 5;

  // Work item = (tile, k-chunk).  Hardware deals workgroups to the 8 XCDs round-robin; XCD x
  // owns a contiguous range of the logical tile order and walks through it once per k-chunk,
  // so that the 32 workgroups resident on an XCD share panels through its L2 and all XCDs are
  // on the same chunk of tokens at the same time.
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int cnt = (a.ntiles >> 3) + (xcd < (a.ntiles & 7) ? 1 : 0);
  if (local >= cnt * a.nsplit) return;  // uniform per workgroup, before any barrier
  const int chunk = local / cnt;
  const int logical = xcd * (a.ntiles >> 3) + min(xcd, a.ntiles & 7) + local % cnt;
  int ti, tj;
  tile_from_index(logical, a.nt, ti, tj);
  const int64_t i0 = (int64_t)ti * kSyTile, j0 = (int64_t)tj * kSyTile;

  // producer: lane -> 8 channels of one token row; lanes 0..31 i-panel, 32..63 j-panel
  const int64_t ch0 = (lane < 32 ? i0 : j0) + 8 * (lane & 31);
  const uint32_t voff = (uint32_t)(ch0 * 2);
  const uint32_t lds_base =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

  // consumer: byte offset of this lane's transposing read inside a stage, fragment 0, slice 0
  const int s16 = lane & 15, g16 = (lane & 31) >> 4;
  const int lane_off = (8 * hi + (s16 >> 2)) * kDmaRow + (16 * g16 + 4 * (s16 & 3)) * 2;

  f32x16 acc[4][GN];
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int g = 0; g < GN; ++g)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[f][g][r] = 0.f;

  const int64_t nkt_all = (a.n_tok + kDmaKT - 1) / kDmaKT;
  const int64_t kbeg = nkt_all * chunk / a.nsplit, nkt = nkt_all * (chunk + 1) / a.nsplit;

  // Descriptor and LDS destination of this wavefront's row loads of k-step kt (scalar
  // registers).  Steps past the end get an empty descriptor: every lane is out of range, nothing
  // is read and zeros are written, so the wait counts below stay uniform.
  auto prep = [&](int64_t kt, u32x4& rs, uint32_t& dst) {
    const int64_t t0 = kt * kDmaKT + RPW * wave;
    int64_t rem_bytes = ((a.n_tok - t0 - 1) * a.ldx + a.b) * 2;
    const uint16_t* base = a.X + t0 * a.ldx;
    if (t0 >= a.n_tok) {
      rem_bytes = 0;
      base = a.X;
    }
    const uint32_t nrec = rem_bytes > 0xffffffffll ? 0xffffffffu : (uint32_t)rem_bytes;
    const uint64_t ba = reinterpret_cast<uint64_t>(base);
    rs.x = __builtin_amdgcn_readfirstlane((uint32_t)ba);
    rs.y = __builtin_amdgcn_readfirstlane((uint32_t)(ba >> 32) & 0xffffu);  // stride 0
    rs.z = __builtin_amdgcn_readfirstlane(nrec);
    rs.w = 0x00020000u;
    dst = __builtin_amdgcn_readfirstlane(
        lds_base + (uint32_t)((int)(kt % kDmaStages) * kDmaStageBytes + (RPW * wave) * kDmaRow));
  };
  const uint32_t row_bytes = __builtin_amdgcn_readfirstlane((uint32_t)(a.ldx * 2));
  auto issue = [&](int64_t kt) {
    u32x4 rs;
    uint32_t dst;
    prep(kt, rs, dst);
#pragma unroll
    for (int r = 0; r < RPW; ++r) dma_row(rs, dst + r * kDmaRow, voff, r * row_bytes);
  };
  // Fragment k of a 16-token slice, in the order the MFMAs first need them:
  // a0, b0 .. b(GN-1), a1, a2, a3.
  auto read_item = [&](int k, const char* st, u32x4 (&af)[4], u32x4 (&bf)[GN]) {
    if (k == 0) af[0] = frag_read_tr(st, (32 * (4 * wm)) * 2);
    else if (k <= GN) bf[k - 1] = frag_read_tr(st, 512 + (32 * (GN * wn + k - 1)) * 2);
    else af[k - GN] = frag_read_tr(st, (32 * (4 * wm + k - GN)) * 2);
  };

  // Schedule per k-step kt (two 16-token slices of NMF MFMAs each):
  //   MFMAs of slice 0, with the fragment reads of slice 1 riding behind the first of them |
  //   wait: own loads of kt+1 landed, own LDS reads done | barrier |
  //   MFMAs of slice 1, with the fragment reads of slice 0 of kt+1 behind the first half and
  //   the row loads of kt+4 (into the stage of kt) behind the second half.
  // All wavefronts of a workgroup leave the barrier together, so anything issued in a bunch
  // there would leave the matrix core idle on every SIMD at once; issued one or two at a time
  // behind an MFMA (32 cycles each) they cost nothing.  The scheduling barriers pin that order.
  // vmcnt(n): at most n of this wavefront's loads still pending.
  constexpr int kWaitPrologue = (RPW * 3 & 15) | ((RPW * 3 >> 4) << 14) | 0x0F70;  // 3 steps pending
  constexpr int kWaitLoop = (RPW * 2 & 15) | ((RPW * 2 >> 4) << 14) | 0x0070;      // 2 steps, lgkm 0
  constexpr int NMF = 4 * GN;                      // MFMAs per slice
  constexpr int NFR = 4 + GN;                      // operand fragments per slice
  constexpr int SLOTS = NMF / 2;                   // MFMAs that carry fragment reads
  constexpr int PER = (NFR + SLOTS - 1) / SLOTS;   // fragment reads behind each of them
  static_assert(RPW <= NMF - SLOTS, "one row load behind each MFMA of the second half");
  issue(kbeg);
  issue(kbeg + 1);
  issue(kbeg + 2);
  issue(kbeg + 3);
  __builtin_amdgcn_s_waitcnt(kWaitPrologue);
  __syncthreads();
  u32x4 a0[4], b0[GN], a1[4], b1[GN];
  {
    const char* st = lds + (int)(kbeg % kDmaStages) * kDmaStageBytes + lane_off;
#pragma unroll
    for (int k = 0; k < NFR; ++k) read_item(k, st, a0, b0);
  }
  for (int64_t kt = kbeg; kt < nkt; ++kt) {
    {
      const char* st = lds + (int)(kt % kDmaStages) * kDmaStageBytes + lane_off + 16 * kDmaRow;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NMF; ++i) {
        acc[i / GN][i % GN] = mfma16<BF16>(a0[i / GN], b0[i % GN], acc[i / GN][i % GN]);
#pragma unroll
        for (int k = i * PER; k < (i + 1) * PER; ++k)
          if (k < NFR) read_item(k, st, a1, b1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_s_waitcnt(kWaitLoop);
    __syncthreads();
    {
      u32x4 rs;
      uint32_t dst;
      prep(kt + 4, rs, dst);
      const char* st = lds + (int)((kt + 1) % kDmaStages) * kDmaStageBytes + lane_off;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NMF; ++i) {
        acc[i / GN][i % GN] = mfma16<BF16>(a1[i / GN], b1[i % GN], acc[i / GN][i % GN]);
#pragma unroll
        for (int k = i * PER; k < (i + 1) * PER; ++k)
          if (k < NFR) read_item(k, st, a0, b0);
        if (i >= SLOTS && i - SLOTS < RPW)
          dma_row(rs, dst + (i - SLOTS) * kDmaRow, voff, (i - SLOTS) * row_bytes);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0), lgkmcnt(0): drain the look-ahead

  // H[i][j] += alpha * acc for i >= j; MFMA row m <-> channel i0 + 32(4wm+f) + m,
  // MFMA column n <-> channel j0 + 32(GN wn+g) + n: 32 lanes write 128 contiguous bytes.
  if (a.nsplit > 1) {
    // several workgroups hold partial sums of this tile: add them with device-scope atomics
    // (no other access to H happens inside this launch)
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int g = 0; g < GN; ++g) {
        const int64_t j = j0 + 32 * (GN * wn + g) + lo;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = 8 * (r >> 2) + 4 * hi + (r & 3);
          const int64_t i = i0 + 32 * (4 * wm + f) + m;
          if (i < a.b && j <= i)
            (void)__hip_atomic_fetch_add(a.H + i * a.b + j, a.alpha * acc[f][g][r],
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    return;
  }
  // per 32x32 MFMA tile: 16 loads, then 16 stores (a load behind a store would wait for it)
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int g = 0; g < GN; ++g) {
      const int64_t j = j0 + 32 * (GN * wn + g) + lo;
      float old[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = 8 * (r >> 2) + 4 * hi + (r & 3);
        const int64_t i = i0 + 32 * (4 * wm + f) + m;
        old[r] = (i < a.b && j <= i) ? a.H[i * a.b + j] : 0.f;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = 8 * (r >> 2) + 4 * hi + (r & 3);
        const int64_t i = i0 + 32 * (4 * wm + f) + m;
        if (i < a.b && j <= i) a.H[i * a.b + j] = old[r] + a.alpha * acc[f][g][r];
      }
    }
}

// Number of k-chunks per tile.  One XCD (32 compute units) works through cnt*S items of
// nkt/S k-steps each, plus a fixed cost per item (pipeline fill, write-out) of about `epi`
// k-steps.  S = 1 keeps the plain read-modify-write (bitwise reproducible); it is given up only
// for a gain of more than 3 %.
static int choose_split(int ntiles, int64_t nkt) {
  const int cnt = (ntiles + 7) / 8;
  const double epi = 12.0;
  auto cost = [&](int S) {
    const int64_t rounds = ((int64_t)cnt * S + 31) / 32;
    return (double)rounds * ((double)nkt / S + epi);
  };
  int best = 1;
  double cbest = cost(1);
  const int smax = (int)std::min<int64_t>(64, nkt / 64);
  for (int S = 2; S <= smax; ++S) {
    const double c = cost(S);
    if (c < cbest * (best == 1 ? 0.97 : 1.0)) {
      cbest = c;
      best = S;
    }
  }
  return best;
}

thanos_status syrk_accumulate(hipStream_t s, float* H, int64_t b, const void* Xc,
                              thanos_dtype xdt, int64_t n_tok, int64_t ldx, float alpha) {
  if (n_tok == 0) return THANOS_OK;
  if (xdt == THANOS_F32) {
    // fp32 calibration data: plain fp32 matrix-core product, lower tiles only.
    const float* X = reinterpret_cast<const float*>(Xc);
    return gemm_f32(s, true, true, b, b, n_tok, alpha, X, ldx, X, ldx, 1.f, H, b, true);
  }
  SyrkArgs a;
  a.H = H;
  a.X = reinterpret_cast<const uint16_t*>(Xc);
  a.b = b;
  a.n_tok = n_tok;
  a.ldx = ldx;
  a.alpha = alpha;
  a.nt = (int)ceil_div(b, kSyTile);
  a.ntiles = a.nt * (a.nt + 1) / 2;
  a.nsplit = 1;
  const bool vec = (reinterpret_cast<uintptr_t>(Xc) % 16 == 0) && (ldx % 8 == 0) && (b % 8 == 0);
  const size_t smem = vec ? (size_t)kDmaStages * kDmaStageBytes            // 136 KB
                          : 2 * kSyOct * 512 * sizeof(u32x4);              // 128 KB
  void (*kern)(SyrkArgs);
  constexpr int kNW = 8;
  if (xdt == THANOS_BF16) kern = vec ? k_syrk16_dma<true, kNW> : k_syrk16<true, false>;
  else kern = vec ? k_syrk16_dma<false, kNW> : k_syrk16<false, false>;
  THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
  unsigned grid = (unsigned)a.ntiles;
  if (vec) {
    a.nsplit = choose_split(a.ntiles, (n_tok + kDmaKT - 1) / kDmaKT);
    grid = 8u * (unsigned)((a.ntiles + 7) / 8) * (unsigned)a.nsplit;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(vec ? 64 * kNW : 256), smem, s, a);
  THANOS_LAUNCH_CHECK();
  return THANOS_OK;
}

}  // namespace thanos
