// Pieces that sit next to the per-layer solve in the whole-model procedure (Algorithm 2):
//  - the activation quantiser that produces X, the quantised model's layer input, when activations
//    are quantised before the weights (Section 5.1: per-token asymmetric, clipping ratio 0.9);
//  - packing of the integer codes into a bit stream.
#include "common.h"

namespace gptaq {

__device__ __forceinline__ float up_bf16_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint16_t up_bf16_rne(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ float up_wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float up_wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// double -> bfloat16 with one rounding (nearest, ties to even): truncate to fp32, keep a sticky bit for what was
// cut off, then round the 24-bit value to 8 bits.
__device__ __forceinline__ uint16_t up_f64_to_bf16(double p) {
  const float f = __double2float_rz(p);
  uint32_t u = __float_as_uint(f);
  if ((double)f != p) u |= 1u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// One wavefront per token.  range = clip * [min(0, min x), max(0, max x)], scale = fp32(range / maxq) (the few
// operations per token in fp64, so that the fp32 scale is the correctly rounded quotient),
// zero = rint(-clip*min/scale), x^ = scale * (clamp(rint(x/scale) + zero) - zero): the rounding of x/scale is decided
// exactly (see below), the product is exact in fp64 and is rounded once to bf16.
__global__ __launch_bounds__(256) void fake_quant_tokens_kernel(const uint16_t* X, uint16_t* Y, int tokens, int n,
                                                                int64_t ldx, int64_t ldy, float maxq, float clip) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (t >= tokens) return;
  const uint16_t* x = X + (int64_t)t * ldx;
  float mn = 0.f, mx = 0.f;
  for (int c = lane; c < n; c += 64) {
    const float v = up_bf16_f32(x[c]);
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
  double lo = (double)up_wave_min(mn) * (double)clip, hi = (double)up_wave_max(mx) * (double)clip;
  if (lo == 0.0 && hi == 0.0) { lo = -1.0; hi = 1.0; }
  const float scale = (float)((hi - lo) / (double)maxq);
  const float zero = (float)rint(-lo / (double)scale);
  for (int c = lane; c < n; c += 64) {
    const float v = up_bf16_f32(x[c]);
    // rint(v / scale), decided exactly: with few-bit inputs and ranges the quotient sits ON a rounding boundary for
    // whole families of values, up to the rounding of the scale, and the rounded fp32 quotient alone cannot tell the
    // side.  The sign of v - (f + 1/2) scale, formed with one rounding by the FMA, can.
    const float f = floorf(v / scale);
    const float side = fmaf(-(f + 0.5f), scale, v);
    const bool odd = ((int)f) & 1;
    const float r = side > 0.f ? f + 1.f : (side < 0.f ? f : (odd ? f + 1.f : f));
    const float q = fminf(fmaxf(r + zero, 0.f), maxq);
    Y[(int64_t)t * ldy + c] = up_f64_to_bf16((double)scale * (double)(q - zero));
  }
}

// Row r of `packed` is the little-endian bit stream of the row's codes: code j occupies bits
// [j*bits, (j+1)*bits).  One thread per 32-bit output word.
__global__ __launch_bounds__(256) void pack_codes_kernel(const uint8_t* codes, int64_t ldc, int m, int n, int bits,
                                                         uint32_t* packed, int64_t words_per_row) {
  const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int r = blockIdx.y;
  if (w >= words_per_row) return;
  const int64_t bit0 = w * 32;
  int64_t j = bit0 / bits;                    // first code that touches this word
  uint32_t out = 0;
  for (; j < n && j * bits < bit0 + 32; ++j) {
    const uint32_t c = codes[(int64_t)r * ldc + j] & ((1u << bits) - 1u);
    const int64_t sh = j * bits - bit0;
    out |= sh >= 0 ? c << sh : c >> (-sh);
  }
  packed[(int64_t)r * words_per_row + w] = out;
}

}  // namespace gptaq

using namespace gptaq;

extern "C" int gptaq_fake_quant_activations(const uint16_t* X, uint16_t* Y, int64_t tokens, int64_t n, int64_t ldx,
                                            int64_t ldy, int bits, float clip, void* stream) {
  if (!X || !Y) return GPTAQ_ENULL;
  if (tokens < 0 || n <= 0 || ldx < n || ldy < n || tokens > ((int64_t)1 << 31) - 8) return GPTAQ_EDIM;
  if (bits < 2 || bits > 16 || !(clip > 0.f && clip <= 1.f)) return GPTAQ_EUNSUPPORTED;
  if (tokens == 0) return GPTAQ_OK;
  hipLaunchKernelGGL(fake_quant_tokens_kernel, dim3((unsigned)((tokens + 3) / 4)), dim3(256), 0, (hipStream_t)stream, X,
                     Y, (int)tokens, (int)n, ldx, ldy, (float)((1 << bits) - 1), clip);
  GPTAQ_LAUNCH_CHECK();
  return GPTAQ_OK;
}

extern "C" int64_t gptaq_packed_words_per_row(int64_t n, int bits) {
  return (n <= 0 || bits < 1 || bits > 8) ? 0 : (n * bits + 31) / 32;
}

extern "C" int gptaq_pack_codes(const uint8_t* codes, int64_t m, int64_t n, int64_t ldc, int bits, uint32_t* packed,
                                void* stream) {
  if (!codes || !packed) return GPTAQ_ENULL;
  if (m <= 0 || n <= 0 || ldc < n || m > 65535 * 64) return GPTAQ_EDIM;
  if (bits < 1 || bits > 8) return GPTAQ_EUNSUPPORTED;
  const int64_t wpr = gptaq_packed_words_per_row(n, bits);
  for (int64_t r0 = 0; r0 < m; r0 += 65535) {
    const int64_t rows = m - r0 < 65535 ? m - r0 : 65535;
    hipLaunchKernelGGL(pack_codes_kernel, dim3((unsigned)((wpr + 255) / 256), (unsigned)rows), dim3(256), 0,
                       (hipStream_t)stream, codes + r0 * ldc, ldc, (int)rows, (int)n, bits, packed + r0 * wpr, wpr);
    GPTAQ_LAUNCH_CHECK();
  }
  return GPTAQ_OK;
}
