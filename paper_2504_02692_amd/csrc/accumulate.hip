// Algorithm 1, line 2:  H += X X^T,  dXXT += (X~ - X) X^T, streamed over token chunks.
//
// Two steps per chunk.  (1) A bandwidth-bound pass reads the token-major bf16 X and X~,
// forms dX = X~ - X in fp32, splits it exactly into two bf16 terms (hi = rne(dX),
// lo = dX - hi) and writes X, hi, lo transposed in k-tile-major order: [token tile of 32]
// [neuron][32 tokens], the operand layout the MFMA GEMM wants (tokens are its K dimension and
// a block of neurons x one token tile is a single contiguous run).
// (2) One launch of the MFMA GEMM computes dXXT += hi X^T + lo X^T on all tiles and
// H += X X^T on the tiles that touch the upper triangle.
#include "common.h"
#include <mutex>

namespace gptaq {

// Workspace of gptaq_accumulate_noalloc: one copy per GPU, owned by the code object, never freed.
constexpr size_t kScratchBytes = (size_t)32 << 20;
constexpr int64_t kScratchMaxN = 16384;                   // 6 * 16384 * 320 tokens still fit
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  __bf16 b = (__bf16)f;                       // v_cvt_pk_bf16_f32: round to nearest even
  return (uint32_t)__builtin_bit_cast(uint16_t, b);
}

// grid: (n_pad / 64, c_pad / 64).  Writes zeros where the source is out of range, so the
// GEMM can run on whole tiles.
__global__ __launch_bounds__(256) void split_transpose_kernel(
    const uint16_t* __restrict__ X, const uint16_t* __restrict__ Xt, int64_t ldx,
    int tokens, int n, uint16_t* __restrict__ oX, uint16_t* __restrict__ oHi,
    uint16_t* __restrict__ oLo, int64_t ldo /* padded rows */, int tile0 /* first 64-token tile of the output */,
    const int32_t* __restrict__ row_of /* NULL, or operand row of input column j (a permutation of 0 .. n-1) */) {
  constexpr int LS = 72;                                  // padded LDS row, 144 bytes
  __shared__ __attribute__((aligned(16))) uint16_t sx[64 * LS], sh[64 * LS], sl[64 * LS];
  const int n0 = blockIdx.x * 64, t0 = blockIdx.y * 64;
  const int tid = threadIdx.x, r = tid >> 3, c = tid & 7;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int t = t0 + r + 32 * p, col = n0 + c * 8;
    u32x4 a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
    if (t < tokens && col < n) {
      a = *reinterpret_cast<const u32x4*>(X + (int64_t)t * ldx + col);
      b = *reinterpret_cast<const u32x4*>(Xt + (int64_t)t * ldx + col);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t xa = (a[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
      const uint32_t xb = (b[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
      const float d = bf16_to_f32(xb) - bf16_to_f32(xa);
      const uint32_t hi = f32_to_bf16_rne(d);
      const uint32_t lo = f32_to_bf16_rne(d - bf16_to_f32(hi));
      const int o = (c * 8 + e) * LS + r + 32 * p;
      sx[o] = (uint16_t)xa;
      sh[o] = (uint16_t)hi;
      sl[o] = (uint16_t)lo;
    }
  }
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int nl = r + 32 * p;
    int64_t row = n0 + nl;                                  // (padding rows stay where they are)
    if (row_of && row < n) {
      const int32_t rr = row_of[row];
      if (rr >= 0 && rr < n) row = rr;                      // (an entry out of range cannot send a write out of bounds)
    }
    const int64_t g = (((int64_t)(blockIdx.y + tile0) * 2 + (c >> 2)) * ldo + row) * 32 + (c & 3) * 8;   // k-tile-major
    *reinterpret_cast<u32x4*>(oX + g) = *reinterpret_cast<const u32x4*>(sx + nl * LS + c * 8);
    *reinterpret_cast<u32x4*>(oHi + g) = *reinterpret_cast<const u32x4*>(sh + nl * LS + c * 8);
    *reinterpret_cast<u32x4*>(oLo + g) = *reinterpret_cast<const u32x4*>(sl + nl * LS + c * 8);
  }
}

__global__ void symmetrize_kernel(float* H, int n, int64_t ldh) {
  __shared__ float t[32][33];
  const int bi = blockIdx.y, bj = blockIdx.x;
  if (bj < bi) return;                                     // handle pairs once, from the upper side
  const int i = bi * 32 + threadIdx.y, j = bj * 32 + threadIdx.x;
  if (i < n && j < n) t[threadIdx.y][threadIdx.x] = H[(int64_t)i * ldh + j];
  __syncthreads();
  const int li = bj * 32 + threadIdx.y, lj = bi * 32 + threadIdx.x;   // transposed position
  if (li < n && lj < n && li > lj) H[(int64_t)li * ldh + lj] = t[threadIdx.x][threadIdx.y];
}

// diag[j] += sum_t X[t][j]^2 (the diagonal of H) for the 32 columns of a workgroup: thread = (token lane, 8 columns),
// 64 token lanes; products of bf16 numbers are exact in fp32, the sums are taken in a fixed order.
__global__ __launch_bounds__(256) void column_sumsq_kernel(const uint16_t* __restrict__ X, int64_t ldx, int tokens, int n,
                                                           float* __restrict__ diag) {
  __shared__ float part[64][33];
  const int oct = threadIdx.x & 3, tl = threadIdx.x >> 2, col = blockIdx.x * 32 + oct * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < n)
    for (int t = tl; t < tokens; t += 64) {
      const u32x4 a = *reinterpret_cast<const u32x4*>(X + (int64_t)t * ldx + col);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = bf16_to_f32((a[e >> 1] >> ((e & 1) * 16)) & 0xffffu);
        acc[e] = fmaf(x, x, acc[e]);
      }
    }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[tl][oct * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < 32 && blockIdx.x * 32 + threadIdx.x < n) {
    float sum = 0.f;
    for (int l = 0; l < 64; ++l) sum += part[l][threadIdx.x];
    diag[blockIdx.x * 32 + threadIdx.x] += sum;
  }
}

__global__ void invert_permutation_kernel(const int32_t* perm, int n, int32_t* inv) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r < n) {
    const int32_t i = perm[r];
    if (i >= 0 && i < n) inv[i] = r;
  }
}

static int64_t padded_n(int64_t n) { return round_up(n, gemm_tile_for(n, n)); }

}  // namespace gptaq

using namespace gptaq;

extern "C" size_t gptaq_accumulate_workspace_bytes(int64_t tokens, int64_t n) {
  if (tokens <= 0 || n <= 0) return 0;
  const int64_t c = round_up(tokens < 32768 ? tokens : 32768, 64);
  return (size_t)(3 * padded_n(n) * c * 2);
}

// H += X X^T (upper tiles) and dXXT += (hi + lo) X^T over cp tokens of split operands, as one launch.
// dxxt_upper: only the tiles of dXXT that touch its upper triangle.  Eq. 17 masks dXXT L to its strictly upper part and
// L is lower triangular, so entry (i, k) of dXXT reaches P only through sums over k >= j > i: in the natural column
// order nothing on or below the diagonal is ever read, and two fifths of the products of the launch can be left out.
static hipError_t launch_products(const uint16_t* oX, const uint16_t* oHi, const uint16_t* oLo, int64_t np, int64_t cp,
                                  int64_t n, float* H, float* dXXT, int64_t ldh, bool dxxt_upper, hipStream_t s) {
  const int tile = gemm_tile_for(n, n);
  GemmBatch b{};
  b.nprob = 2;
  b.tile = tile;
  GemmProblem& a = b.p[0];
  a.C = dXXT; a.ldc = ldh; a.M = (int)n; a.N = (int)n; a.K = (int)cp;
  a.tiles_m = a.tiles_n = (int)(np / tile);
  a.kind = 1; a.nterm = 1; a.tile_mode = dxxt_upper ? 2 : 0; a.k_mode = 0; a.store_mode = 0;
  a.term[0] = {{oHi, oLo}, {oX, oX}, 32, 32, np * 32, np * 32};
  GemmProblem& h = b.p[1];
  h = a;
  h.C = H; h.kind = 0; h.tile_mode = 2;
  h.term[0] = {{oX, oX}, {oX, oX}, 32, 32, np * 32, np * 32};
  ProfScope ps(kProfAccumGemm, s);
  return launch_gemm(b, s);
}

// the argument checks that need no workspace
static int accumulate_args(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n, int64_t ldx, float* H,
                           float* dXXT, int64_t ldh) {
  if (!X || !Xtilde || !H || !dXXT) return GPTAQ_ENULL;
  if (tokens < 0 || n <= 0 || n % 8 || ldx < n || ldx % 8 || ldh < n || n > (1 << 20) ||
      tokens > (int64_t)1 << 30)
    return GPTAQ_EDIM;
  if (((uintptr_t)X | (uintptr_t)Xtilde) & 15) return GPTAQ_EDIM;
  return GPTAQ_OK;
}

static int accumulate_impl(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n, int64_t ldx, float* H,
                           float* dXXT, int64_t ldh, bool dxxt_upper, void* ws, size_t ws_bytes, void* stream,
                           const int32_t* row_of = nullptr) {
  if (!ws) return GPTAQ_ENULL;
  if (const int rc = accumulate_args(X, Xtilde, tokens, n, ldx, H, dXXT, ldh)) return rc;
  if ((uintptr_t)ws & 255) return GPTAQ_EWORKSPACE;
  if (tokens == 0) return GPTAQ_OK;
  hipStream_t s = (hipStream_t)stream;
  const int64_t np = padded_n(n);
  int64_t cmax = (int64_t)(ws_bytes / (size_t)(6 * np)) / 64 * 64;
  if (cmax < 64) return GPTAQ_EWORKSPACE;
  if (cmax > 32768) cmax = 32768;    // keeps one fp32 running sum short (accuracy), and K in int32
  for (int64_t t0 = 0; t0 < tokens; t0 += cmax) {
    const int64_t c = tokens - t0 < cmax ? tokens - t0 : cmax;
    const int64_t cp = round_up(c, 64);
    uint16_t* oX = (uint16_t*)ws;
    uint16_t* oHi = oX + np * cp;
    uint16_t* oLo = oHi + np * cp;
    {
      ProfScope ps(kProfAccumSplit, s);
      hipLaunchKernelGGL(split_transpose_kernel, dim3((unsigned)(np / 64), (unsigned)(cp / 64)),
                         dim3(256), 0, s, X + t0 * ldx, Xtilde + t0 * ldx, ldx, (int)c, (int)n,
                         oX, oHi, oLo, np, 0, row_of);
    }
    GPTAQ_LAUNCH_CHECK();
    hipError_t e = launch_products(oX, oHi, oLo, np, cp, n, H, dXXT, ldh, dxxt_upper, s);
    if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
  }
  return GPTAQ_OK;
}

extern "C" int gptaq_accumulate(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens,
                                int64_t n, int64_t ldx, float* H, float* dXXT, int64_t ldh,
                                void* ws, size_t ws_bytes, void* stream) {
  return accumulate_impl(X, Xtilde, tokens, n, ldx, H, dXXT, ldh, false, ws, ws_bytes, stream);
}

extern "C" int gptaq_accumulate_upper_permuted(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                                               int64_t ldx, const int32_t* inv_perm, float* H, float* dXXT, int64_t ldh,
                                               void* ws, size_t ws_bytes, void* stream) {
  if (!inv_perm) return GPTAQ_ENULL;
  return accumulate_impl(X, Xtilde, tokens, n, ldx, H, dXXT, ldh, true, ws, ws_bytes, stream, inv_perm);
}

extern "C" int gptaq_accumulate_diag(const uint16_t* X, int64_t tokens, int64_t n, int64_t ldx, float* diag, void* stream) {
  if (!X || !diag) return GPTAQ_ENULL;
  if (tokens < 0 || n <= 0 || n % 8 || ldx < n || ldx % 8 || n > (1 << 20) || tokens > (int64_t)1 << 30) return GPTAQ_EDIM;
  if ((uintptr_t)X & 15) return GPTAQ_EDIM;
  if (tokens == 0) return GPTAQ_OK;
  hipLaunchKernelGGL(column_sumsq_kernel, dim3((unsigned)((n + 31) / 32)), dim3(256), 0, (hipStream_t)stream, X, ldx,
                     (int)tokens, (int)n, diag);
  GPTAQ_LAUNCH_CHECK();
  return GPTAQ_OK;
}

extern "C" int gptaq_invert_permutation(const int32_t* perm, int64_t n, int32_t* inv, void* stream) {
  if (!perm || !inv) return GPTAQ_ENULL;
  if (n <= 0 || n > (1 << 24)) return GPTAQ_EDIM;
  hipLaunchKernelGGL(invert_permutation_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, perm,
                     (int)n, inv);
  GPTAQ_LAUNCH_CHECK();
  return GPTAQ_OK;
}

extern "C" int gptaq_accumulate_upper(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens,
                                      int64_t n, int64_t ldx, float* H, float* dXXT, int64_t ldh,
                                      void* ws, size_t ws_bytes, void* stream) {
  return accumulate_impl(X, Xtilde, tokens, n, ldx, H, dXXT, ldh, true, ws, ws_bytes, stream);
}

// Device address of this GPU's copy of `scratch`, looked up once per device (with that device current).
// In host code the array's name is only a handle for this lookup, never an address to hand to a kernel.
static void* scratch_of_current_device() {
  static std::mutex mu;
  static void* ptr[64] = {nullptr};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { set_last_hip_error(e); return nullptr; }
    ptr[dev] = p;
  }
  return ptr[dev];
}

extern "C" int gptaq_accumulate_noalloc(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                                        int64_t ldx, float* H, float* dXXT, int64_t ldh, void* stream) {
  if (const int rc = accumulate_args(X, Xtilde, tokens, n, ldx, H, dXXT, ldh)) return rc;
  if (n > kScratchMaxN) return GPTAQ_ETOOLARGE;
  if (tokens == 0) return GPTAQ_OK;
  void* ws = scratch_of_current_device();
  if (!ws) return GPTAQ_ELAUNCH;
  // every pass overwrites the part of the scratch it reads (zero padding included), so nothing of the last
  // call's contents is ever read and nothing has to be cleared
  return accumulate_impl(X, Xtilde, tokens, n, ldx, H, dXXT, ldh, false, ws, kScratchBytes, stream);
}

static int accumulate_staged_impl(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n, int64_t ldx,
                                  float* H, float* dXXT, int64_t ldh, bool dxxt_upper, void* ws, size_t ws_bytes,
                                  int64_t* pending, int flush, void* stream) {
  constexpr int64_t CAP = 32768;                 // tokens per product launch
  if (!H || !dXXT || !ws || !pending || (tokens > 0 && (!X || !Xtilde))) return GPTAQ_ENULL;
  if (tokens < 0 || n <= 0 || n % 8 || ldx < n || ldx % 8 || ldh < n || n > (1 << 20) || tokens > (int64_t)1 << 30 ||
      *pending < 0 || *pending >= CAP || *pending % 64 || (!flush && tokens % 64))
    return GPTAQ_EDIM;
  if (tokens > 0 && (((uintptr_t)X | (uintptr_t)Xtilde) & 15)) return GPTAQ_EDIM;
  const int64_t np = padded_n(n);
  if (((uintptr_t)ws & 255) || ws_bytes < (size_t)(6 * np * CAP)) return GPTAQ_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  uint16_t *oX = (uint16_t*)ws, *oHi = oX + np * CAP, *oLo = oHi + np * CAP;
  auto products = [&](int64_t cp) { return launch_products(oX, oHi, oLo, np, cp, n, H, dXXT, ldh, dxxt_upper, s); };
  int64_t done = 0, pend = *pending;
  while (done < tokens) {
    const int64_t take = tokens - done < CAP - pend ? tokens - done : CAP - pend, cp = round_up(take, 64);
    {
      ProfScope ps(kProfAccumSplit, s);
      hipLaunchKernelGGL(split_transpose_kernel, dim3((unsigned)(np / 64), (unsigned)(cp / 64)), dim3(256), 0, s,
                         X + done * ldx, Xtilde + done * ldx, ldx, (int)take, (int)n, oX, oHi, oLo, np, (int)(pend / 64), (const int32_t*)nullptr);
    }
    GPTAQ_LAUNCH_CHECK();
    done += take;
    pend += cp;                                    // (only the chunk that comes with flush may be ragged: it is the last)
    if (pend >= CAP) {
      hipError_t e = products(CAP);
      if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
      pend = 0;
    }
  }
  if (flush && pend > 0) {
    hipError_t e = products(pend);
    if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
    pend = 0;
  }
  *pending = pend;
  return GPTAQ_OK;
}

extern "C" int gptaq_accumulate_staged(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n, int64_t ldx,
                                       float* H, float* dXXT, int64_t ldh, void* ws, size_t ws_bytes, int64_t* pending,
                                       int flush, void* stream) {
  return accumulate_staged_impl(X, Xtilde, tokens, n, ldx, H, dXXT, ldh, false, ws, ws_bytes, pending, flush, stream);
}

extern "C" int gptaq_accumulate_staged_upper(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                                             int64_t ldx, float* H, float* dXXT, int64_t ldh, void* ws, size_t ws_bytes,
                                             int64_t* pending, int flush, void* stream) {
  return accumulate_staged_impl(X, Xtilde, tokens, n, ldx, H, dXXT, ldh, true, ws, ws_bytes, pending, flush, stream);
}

extern "C" int gptaq_symmetrize(float* H, int64_t n, int64_t ldh, void* stream) {
  if (!H) return GPTAQ_ENULL;
  if (n <= 0 || ldh < n || n > (1 << 20)) return GPTAQ_EDIM;
  const unsigned g = (unsigned)((n + 31) / 32);
  hipLaunchKernelGGL(symmetrize_kernel, dim3(g, g), dim3(32, 32), 0, (hipStream_t)stream, H, (int)n, ldh);
  GPTAQ_LAUNCH_CHECK();
  return GPTAQ_OK;
}
