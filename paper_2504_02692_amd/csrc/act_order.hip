// act_order (Section 5.2 and 5.3 "weight-only"): process the input channels in the order of decreasing
// Hessian diagonal.  The solve itself is unchanged: the caller permutes H, dXXT and the columns of W
// with the kernels below, runs prepare / quantize_layer on the permuted problem and scatters the
// results back.
#include "common.h"

namespace gptaq {

// perm[r] = i, r = number of inputs that come before i: larger diagonal first, equal diagonals by index.
__global__ __launch_bounds__(256) void rank_diag_kernel(const float* H, int64_t ldh, int n, int32_t* perm) {
  __shared__ float d[256];
  const int i = blockIdx.x * 256 + threadIdx.x;
  const float di = i < n ? H[(int64_t)i * ldh + i] : 0.f;
  int rank = 0;
  for (int j0 = 0; j0 < n; j0 += 256) {
    const int j = j0 + threadIdx.x;
    __syncthreads();
    d[threadIdx.x] = j < n ? H[(int64_t)j * ldh + j] : 0.f;
    __syncthreads();
    const int lim = min(256, n - j0);
    for (int t = 0; t < lim; ++t) {
      const float dj = d[t];
      rank += (dj > di || (dj == di && j0 + t < i)) ? 1 : 0;
    }
  }
  if (i < n) perm[rank] = i;
}

// out[i][j] = in[perm[i]][perm[j]]: a workgroup gathers within one source row (the row stays in L2).
__global__ __launch_bounds__(256) void permute_square_kernel(const float* in, float* out, int n, int64_t ldin,
                                                             int64_t ldout, const int32_t* perm) {
  const int j = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y;
  if (j >= n) return;
  out[(int64_t)i * ldout + j] = in[(int64_t)perm[i] * ldin + perm[j]];
}

__global__ void copy2d_kernel(const float* in, float* out, int n, int64_t ldin, int64_t ldout) {
  const int j = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y;
  if (j < n) out[(int64_t)i * ldout + j] = in[(int64_t)i * ldin + j];
}

// inverse == 0: out[r][i] = in[r][perm[i]] (gather);  inverse != 0: out[r][perm[i]] = in[r][i] (scatter back)
template <typename T>
__global__ __launch_bounds__(256) void permute_columns_kernel(const T* in, T* out, int m, int n, int64_t ldin,
                                                              int64_t ldout, const int32_t* perm, int inverse) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int p = perm[i];
  for (int r = blockIdx.y; r < m; r += gridDim.y) {
    if (inverse) out[(int64_t)r * ldout + p] = in[(int64_t)r * ldin + i];
    else out[(int64_t)r * ldout + i] = in[(int64_t)r * ldin + p];
  }
}

}  // namespace gptaq

using namespace gptaq;

extern "C" int gptaq_act_order(const float* H, int64_t n, int64_t ldh, int32_t* perm, void* stream) {
  if (!H || !perm) return GPTAQ_ENULL;
  if (n <= 0 || (ldh != 0 && ldh < n) || n > (1 << 20)) return GPTAQ_EDIM;     // ldh == 0: H is the diagonal itself
  hipLaunchKernelGGL(rank_diag_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, H, ldh,
                     (int)n, perm);
  GPTAQ_LAUNCH_CHECK();
  return GPTAQ_OK;
}

extern "C" size_t gptaq_permute_hessian_workspace_bytes(int64_t n) { return n > 0 ? (size_t)n * n * 4 : 0; }

extern "C" int gptaq_permute_hessian(float* H, float* dXXT, int64_t n, int64_t ldh, const int32_t* perm, void* ws,
                                     size_t ws_bytes, void* stream) {
  if (!H || !dXXT || !perm || !ws) return GPTAQ_ENULL;
  if (n <= 0 || ldh < n || n > 65535) return GPTAQ_EDIM;
  if (((uintptr_t)ws & 255) || ws_bytes < (size_t)n * n * 4) return GPTAQ_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  float* tmp = (float*)ws;
  const dim3 grid((unsigned)((n + 255) / 256), (unsigned)n);
  // H arrives as its upper triangle: mirror it first, so that the gather never has to read a column
  const int st = gptaq_symmetrize(H, n, ldh, stream);
  if (st != GPTAQ_OK) return st;
  for (int which = 0; which < 2; ++which) {
    float* M = which ? dXXT : H;
    hipLaunchKernelGGL(permute_square_kernel, grid, dim3(256), 0, s, M, tmp, (int)n, ldh, n, perm);
    GPTAQ_LAUNCH_CHECK();
    hipLaunchKernelGGL(copy2d_kernel, grid, dim3(256), 0, s, tmp, M, (int)n, n, ldh);
    GPTAQ_LAUNCH_CHECK();
  }
  return GPTAQ_OK;
}

template <typename T>
static int permute_columns(const T* in, T* out, int64_t m, int64_t n, int64_t ldin, int64_t ldout, const int32_t* perm,
                           int inverse, void* stream) {
  if (!in || !out || !perm) return GPTAQ_ENULL;
  if (m <= 0 || n <= 0 || ldin < n || ldout < n || (const void*)in == (const void*)out || n > (1 << 24)) return GPTAQ_EDIM;
  const unsigned gy = (unsigned)(m < 4096 ? m : 4096);
  hipLaunchKernelGGL((permute_columns_kernel<T>), dim3((unsigned)((n + 255) / 256), gy), dim3(256), 0,
                     (hipStream_t)stream, in, out, (int)m, (int)n, ldin, ldout, perm, inverse);
  GPTAQ_LAUNCH_CHECK();
  return GPTAQ_OK;
}

extern "C" int gptaq_permute_columns_f32(const float* in, float* out, int64_t m, int64_t n, int64_t ldin, int64_t ldout,
                                         const int32_t* perm, int inverse, void* stream) {
  return permute_columns<float>(in, out, m, n, ldin, ldout, perm, inverse, stream);
}

extern "C" int gptaq_permute_columns_u8(const uint8_t* in, uint8_t* out, int64_t m, int64_t n, int64_t ldin,
                                        int64_t ldout, const int32_t* perm, int inverse, void* stream) {
  return permute_columns<uint8_t>(in, out, m, n, ldin, ldout, perm, inverse, stream);
}
