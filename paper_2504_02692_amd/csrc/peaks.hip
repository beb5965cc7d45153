// Measured ceiling of the bf16 matrix cores: a loop of nothing but independent v_mfma_f32_32x32x16_bf16 on
// every CU, operands held in registers.  The sustained rate depends on the operand data (the chip is
// power-limited: more toggling bits, lower clock), so the caller picks constant or random operands; the
// random ones are the fair ceiling for a GEMM on real data.
#include "common.h"

namespace gptaq {

__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, int random_data, float* sink, unsigned long long* clk) {
  u32x4 ra[8], rb[8];
  uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      s = s * 1664525u + 1013904223u; const uint32_t x = s;
      s = s * 1664525u + 1013904223u; const uint32_t y = s;
      // pairs of bf16 in [1, 2) and (-2, -1]: random sign and mantissa, or all 1.0
      ra[i][v] = random_data ? ((x & 0x807f807fu) | 0x3f803f80u) : 0x3f803f80u;
      rb[i][v] = random_data ? ((y & 0x807f807fu) | 0x3f803f80u) : 0x3f803f80u;
    }
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  const unsigned long long c0 = __builtin_readcyclecounter(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ra[i]), __builtin_bit_cast(bf16x8, rb[(i + u) & 7]),
                                                         acc[i], 0, 0, 0);
  }
  const unsigned long long c1 = __builtin_readcyclecounter(), w1 = wall_clock64();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) t += acc[i][v];
  sink[blockIdx.x * 256 + threadIdx.x] = t;
  if (blockIdx.x == 0 && threadIdx.x == 0) { clk[0] = c1 - c0; clk[1] = w1 - w0; }
}

// Streaming copy: every thread moves 16-byte pieces a whole grid apart, reads and writes fully coalesced.
__global__ __launch_bounds__(256) void stream_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace gptaq

using namespace gptaq;

extern "C" int gptaq_measure_mfma_peak(int random_data, int millis, void* ws, size_t ws_bytes, double* tflops,
                                       double* clock_ghz, void* stream) {
  if (!ws || !tflops || !clock_ghz) return GPTAQ_ENULL;
  if (millis <= 0 || millis > 2000) return GPTAQ_EDIM;
  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return GPTAQ_ELAUNCH;
  const int wgs = prop.multiProcessorCount;               // one workgroup of four wavefronts per CU
  if (((uintptr_t)ws & 255) || ws_bytes < (size_t)wgs * 256 * 4 + 256) return GPTAQ_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  float* sink = (float*)ws;
  unsigned long long* clk = (unsigned long long*)((unsigned char*)ws + (size_t)wgs * 256 * 4);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return GPTAQ_ELAUNCH;
  // a 32-MFMA trip takes about 1024 clocks: ~2000 trips per millisecond; one untimed launch first
  const int iters = millis * 2000;
  float ms = 0.f;
  for (int rep = 0; rep < 2; ++rep) {
    hipEventRecord(e0, s);
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(wgs), dim3(256), 0, s, iters, random_data, sink, clk);
    hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
      set_last_hip_error(hipGetLastError());
      hipEventDestroy(e0); hipEventDestroy(e1);
      return GPTAQ_ELAUNCH;
    }
  }
  unsigned long long h[2] = {0, 1};
  hipError_t e = hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost);
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
  const double flop = (double)wgs * 4 * iters * 32 * (32.0 * 32 * 16 * 2);
  *tflops = flop / (ms * 1e-3) / 1e12;
  *clock_ghz = (double)h[0] / ((double)h[1] * 10.0);      // shader clocks per 100 MHz real-time tick
  return GPTAQ_OK;
}

extern "C" int gptaq_measure_hbm_copy(size_t bytes, int reps, void* ws, size_t ws_bytes, double* gbps, void* stream) {
  if (!ws || !gbps) return GPTAQ_ENULL;
  if (bytes < 4096 || bytes % 16 || reps <= 0 || reps > 1000) return GPTAQ_EDIM;
  if (((uintptr_t)ws & 255) || ws_bytes < 2 * bytes) return GPTAQ_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const u32x4* src = (const u32x4*)ws;
  u32x4* dst = (u32x4*)((unsigned char*)ws + bytes);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return GPTAQ_ELAUNCH;
  const size_t n16 = bytes / 16;
  const unsigned grid = (unsigned)((n16 + 256 * 8 - 1) / (256 * 8) < 65536 * 16 ? (n16 + 256 * 8 - 1) / (256 * 8) : 65536 * 16);
  float ms = 0.f;
  hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(256), 0, s, src, dst, n16);      // untimed
  hipEventRecord(e0, s);
  for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(256), 0, s, src, dst, n16);
  hipEventRecord(e1, s);
  const bool ok = hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  hipEventDestroy(e0); hipEventDestroy(e1);
  if (!ok || hipGetLastError() != hipSuccess) { set_last_hip_error(hipGetLastError()); return GPTAQ_ELAUNCH; }
  *gbps = 2.0 * (double)bytes * reps / (ms * 1e-3) / 1e9;
  return GPTAQ_OK;
}
