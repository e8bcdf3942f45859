// Measured ceilings of the chip the library runs on (gfx950), for reading the roofline
// fractions of the kernels against what the hardware sustains rather than the data sheet:
//   * dense fp16 matrix-core rate of a loop that issues nothing but v_mfma_f32_32x32x16_f16
//     (no loads, no LDS), two wavefronts per SIMD on every compute unit, with the shader clock
//     the chip grants while it runs (cycle counter against the 100 MHz wall clock);
//   * HBM copy bandwidth (read + write of a large buffer).
// Stand-alone C ABI (libthanos_probe.so); nothing in libthanos depends on it.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// out[2*wg + 0] = shader cycles, + 1 = 10 ns ticks of the wall clock (thread 0 of the
// workgroup).  RANDOM: every MFMA of the loop body has operands of its own, pseudo-random fp16
// values in (-2, 2) that differ from lane to lane, so that the multiplier inputs toggle from one
// MFMA to the next as they do on real data (the power a matrix core draws, hence the clock the
// chip grants, depends on it); otherwise all MFMAs share one smooth operand pair.
template <bool RANDOM>
__global__ __launch_bounds__(512, 2) void k_mfma_only(int iters, unsigned int seed, float* sink,
                                                       unsigned long long* out) {
  constexpr int NACC = 8;  // independent accumulators: 8 MFMAs of 32 cycles between reuses
  f32x16 acc[NACC];
  f16x8 a[NACC], b[NACC];
  unsigned int x = seed * 2654435761u + threadIdx.x * 40503u + blockIdx.x * 9973u + 12345u;
#pragma unroll
  for (int k = 0; k < NACC; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (RANDOM) {
        x = x * 1664525u + 1013904223u;
        a[k][e] = (_Float16)(((int)(x >> 8 & 0xffff) - 32768) * (1.f / 16384.f));
        x = x * 1664525u + 1013904223u;
        b[k][e] = (_Float16)(((int)(x >> 8 & 0xffff) - 32768) * (1.f / 16384.f));
      } else {
        a[k][e] = (_Float16)(1.0f + 0.001f * (threadIdx.x & 7) + 0.01f * e);
        b[k][e] = (_Float16)(0.5f - 0.002f * e);
      }
    }
#pragma unroll
  for (int k = 0; k < NACC; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < NACC; ++k)
      acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[k], b[k], acc[k], 0, 0, 0);
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < NACC; ++k)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[k][r];
  if (s == 12345.678f) sink[0] = s;  // practically never true; the compiler cannot know
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x + 0] = (unsigned long long)(c1 - c0);
    out[2 * blockIdx.x + 1] = (unsigned long long)(w1 - w0);
  }
}

__global__ __launch_bounds__(256) void k_copy16(const uint4* __restrict__ src,
                                                uint4* __restrict__ dst, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
    dst[i] = src[i];
}

extern "C" {

// Runs the MFMA-only loop on `wgs` workgroups of 8 wavefronts for `iters` iterations of 8 MFMAs
// per wavefront, with smooth shared operands (random_operands = 0) or per-MFMA pseudo-random ones.  Host outputs: ms (launch duration by events), tflops, shader clock in GHz
// (mean over the workgroups).  scratch: device buffer of at least 16 * wgs + 16 bytes.
// Returns 0, or a HIP error code.
int thanos_probe_mfma_f16(int wgs, int iters, int random_operands, void* scratch, double* ms,
                          double* tflops, double* sclk_ghz, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  unsigned long long* out = (unsigned long long*)scratch;
  float* sink = (float*)(out + 2 * (size_t)wgs);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
  auto launch = [&](int n) {
    if (random_operands)
      hipLaunchKernelGGL(k_mfma_only<true>, dim3(wgs), dim3(512), 0, s, n, 7u, sink, out);
    else
      hipLaunchKernelGGL(k_mfma_only<false>, dim3(wgs), dim3(512), 0, s, n, 7u, sink, out);
  };
  launch(64);  // warm-up
  (void)hipEventRecord(e0, s);
  launch(iters);
  (void)hipEventRecord(e1, s);
  hipError_t err = hipEventSynchronize(e1);
  if (err != hipSuccess) return (int)err;
  float t = 0.f;
  (void)hipEventElapsedTime(&t, e0, e1);
  unsigned long long* h = new unsigned long long[2 * (size_t)wgs];
  err = hipMemcpy(h, out, 16 * (size_t)wgs, hipMemcpyDeviceToHost);
  double cyc = 0, tick = 0;
  for (int i = 0; i < wgs; ++i) {
    cyc += (double)h[2 * i];
    tick += (double)h[2 * i + 1];
  }
  delete[] h;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *ms = t;
  // 8 wavefronts x iters x 8 MFMAs x (32 x 32 x 16 x 2 flops)
  *tflops = (double)wgs * 8.0 * iters * 8.0 * 32768.0 / (t * 1e-3) / 1e12;
  *sclk_ghz = tick > 0 ? cyc / (tick * 10.0) : 0.0;  // cycles per 10 ns -> GHz
  return (int)err;
}

// Copies `bytes` (multiple of 16) from src to dst `reps` times; gbs = (read + written) / time.
int thanos_probe_copy(const void* src, void* dst, int64_t bytes, int reps, double* ms, double* gbs,
                      void* stream) {
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
  const int64_t n = bytes / 16;
  hipLaunchKernelGGL(k_copy16, dim3(8192), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
  (void)hipEventRecord(e0, s);
  for (int r = 0; r < reps; ++r)
    hipLaunchKernelGGL(k_copy16, dim3(8192), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, n);
  (void)hipEventRecord(e1, s);
  hipError_t err = hipEventSynchronize(e1);
  float t = 0.f;
  (void)hipEventElapsedTime(&t, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *ms = t / reps;
  *gbs = 2.0 * (double)bytes / (t / reps * 1e-3) / 1e9;
  return (int)err;
}

}  // extern "C"
