// thanos_hessian_accumulate: H += alpha * Xc^T Xc on the CDNA4 matrix cores.
//
// Xc is token-major [n_tok, b] (16-bit floats), so both MFMA operands of H = Xc^T Xc are
// "channel-contiguous": the reduction index (token) is the strided one.  The 16-bit MFMA wants
// 8 consecutive reduction values per lane in 4 VGPRs, so every 8-token x 8-channel patch is
// transposed in registers (v_perm_b32) on its way from global memory to LDS.  Two freedoms of a
// Gram matrix make the LDS traffic conflict-free in both directions:
//   * the order of the reduction index is arbitrary as long as both operands use the same one;
//   * a 32-row MFMA operand may be ANY 32 channels: fragment f of a 256-channel panel is
//     {8x + f : x = 0..31}, which is exactly what 32 lanes hold after the register transpose.
//
// Workgroup = 256 threads = 4 wavefronts (2x2), tile = 256 x 256 outputs, each wavefront
// 128 x 128 = 4x4 MFMA 32x32x16 tiles (256 accumulator registers).  A k-step is 64 tokens:
// 8 octets of 8 tokens; LDS stage = 8 octets x 512 channel slots x 16 B = 64 KB, two stages.
// Only tiles on or below the diagonal are computed.  Workgroups are renumbered so that the 32
// workgroups resident on one XCD work on a 4 x 8 patch of neighbouring tiles and share their
// panels of X through that XCD's L2.
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
  const bool vec = (reinterpret_cast<uintptr_t>(Xc) % 16 == 0) && (ldx % 8 == 0) && (b % 8 == 0);
  const size_t smem = 2 * kSyOct * 512 * sizeof(u32x4);  // 128 KB
  void (*kern)(SyrkArgs);
  if (xdt == THANOS_BF16) kern = vec ? k_syrk16<true, true> : k_syrk16<true, false>;
  else kern = vec ? k_syrk16<false, true> : k_syrk16<false, false>;
  THANOS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
  hipLaunchKernelGGL(kern, dim3((unsigned)a.ntiles), dim3(256), smem, s, a);
  THANOS_LAUNCH_CHECK();
  return THANOS_OK;
}

}  // namespace thanos
