// Algorithm 1, lines 3-4: damping, the inverse-Cholesky factor and the fused matrix P.
//
// Step 3 of the paper needs L with (H + lambda I)^-1 = L L^T.  Instead of inverting and then
// factoring, factor  H + lambda I = V V^T  with V UPPER triangular (a Cholesky factorisation
// run from the last row/column towards the first); then U = L^T = V^-1 (the factor is unique
// for a positive diagonal).  Both the factorisation and the triangular inverse are swept
// from the bottom-right block to the top-left block in one pass, in fp64, 64 columns at a
// time, inside one n x n fp64 array F:
//
//   for K = last block .. first block                       (I: blocks above K, J: other blocks)
//     diag   : F_KK = V_KK V_KK^T,  Winv = V_KK^-1,  U_KK = Winv
//     panel  : V_IK = F_IK Winv^T            (rows above)   } one launch
//     rowblk : U_KJ = Winv R_KJ              (J right of K) }
//     update : F_IJ -= V_IK V_JK^T  (I <= J < K, Schur complement)
//              R_IJ -= V_IK U_KJ    (J > K, right-looking solve of V U = I)
//     close  : R_IK  = -V_IK U_KK
//
// The strictly-upper region of F holds Schur-complement data until its block column is
// factored and the running right-hand side R of the triangular solve afterwards, so no
// second n x n array is needed.  Theorem 4.2's two products then run on the MFMA GEMM with
// fp32 operands split into bf16 hi+lo (three cross products per term).
#include "common.h"

namespace gptaq {

constexpr int NB = 64;
constexpr int LDT = 65;                       // padded LDS row (doubles)
constexpr int MM_LDS = 2 * NB * LDT * 8;      // bytes for two staged tiles

struct Sweep {
  double* F;
  int64_t ldf;
  int n, kb, nblk;
  double* Dinv;      // nblk tiles of 64 x 64: V_KK^-1
  int32_t* info;
};

// ----------------------------------------------------------------------------- statistics
// One workgroup: dead inputs, lambda = damp * mean(diag), info words.
__global__ __launch_bounds__(1024) void diag_stats_kernel(const float* H, int64_t ldh, int n, float damp,
                                                          uint8_t* dead, double* lam_out, int32_t* info) {
  __shared__ double ssum[1024];
  __shared__ int scnt[1024];
  double s = 0.0;
  int c = 0;
  for (int i = threadIdx.x; i < n; i += 1024) {
    float d = H[(int64_t)i * ldh + i];
    const bool dd = d == 0.f;
    if (dd) { d = 1.f; ++c; }
    if (dead) dead[i] = dd ? 1 : 0;
    s += (double)d;
  }
  ssum[threadIdx.x] = s;
  scnt[threadIdx.x] = c;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) { ssum[threadIdx.x] += ssum[threadIdx.x + o]; scnt[threadIdx.x] += scnt[threadIdx.x + o]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *lam_out = (double)damp * ssum[0] / (double)n;
    info[0] = 0;
    info[1] = scnt[0];
  }
}

// F (upper triangle, fp64) = H + lambda I with the dead-input rule applied.
__global__ void build_F_kernel(const float* H, int64_t ldh, int n, const double* lam, double* F, int64_t ldf) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x, i = blockIdx.y;
  if (j >= n || j < i) return;
  double v = (double)H[(int64_t)i * ldh + j];
  if (i == j) { if (v == 0.0) v = 1.0; v += *lam; }
  F[(int64_t)i * ldf + j] = v;
}

// ------------------------------------------------------------------- 64 x 64 x 64 in LDS
// out[i][c] = sum_l A[i][l] * B[l][c] with As[l*LDT + i], Bs[l*LDT + c]; thread (ty, tx)
// owns rows 4ty..4ty+3 and columns tx + 16q.
__device__ __forceinline__ void mm64(const double* As, const double* Bs, double acc[4][4]) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[p][q] = 0.0;
#pragma unroll 4
  for (int l = 0; l < NB; ++l) {
    double a[4], b[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) a[p] = As[l * LDT + 4 * ty + p];
#pragma unroll
    for (int q = 0; q < 4; ++q) b[q] = Bs[l * LDT + tx + 16 * q];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[p][q] = fma(a[p], b[q], acc[p][q]);
  }
}

// Stage a 64 x 64 tile of a row-major fp64 matrix.  transposed == false: dst[c*LDT + r] = src[r][c]
// ("k-major A": r is the output row, c the contraction index).  transposed == true:
// dst[r*LDT + c] = src[r][c].  Out-of-range elements read as 0.
__device__ __forceinline__ void stage_tile(double* dst, const double* src, int64_t ld, int r0, int c0,
                                           int rmax, int cmax, bool row_major_dst) {
  const int c = threadIdx.x & 63, rb = threadIdx.x >> 6;
#pragma unroll 4
  for (int p = 0; p < 16; ++p) {
    const int r = rb + 4 * p;
    double v = 0.0;
    if (r0 + r < rmax && c0 + c < cmax) v = src[(int64_t)(r0 + r) * ld + c0 + c];
    if (row_major_dst) dst[r * LDT + c] = v; else dst[c * LDT + r] = v;
  }
}

// ------------------------------------------------------------------------------- diag
__global__ __launch_bounds__(256) void diag_kernel(Sweep a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  double* S = reinterpret_cast<double*>(smem_raw);        // S[r*LDT + c]
  double* Wi = S + NB * LDT;
  const int tid = threadIdx.x;
  const int k0 = a.kb * NB, w = min(NB, a.n - k0);
  // load the upper triangle, mirror it, identity in the padding
  for (int idx = tid; idx < NB * NB; idx += 256) {
    const int r = idx >> 6, c = idx & 63;
    double v;
    if (r < w && c < w) {
      const int rr = min(r, c), cc = max(r, c);
      v = a.F[(int64_t)(k0 + rr) * a.ldf + k0 + cc];
    } else {
      v = r == c ? 1.0 : 0.0;
    }
    S[r * LDT + c] = v;
    Wi[r * LDT + c] = 0.0;
  }
  const int ti = tid >> 4, tl = tid & 15;
  for (int j = NB - 1; j >= 0; --j) {
    __syncthreads();
    const double sjj = S[j * LDT + j];
    const bool bad = !(sjj > 0.0);
    const double d = bad ? 1.0 : sqrt(sjj);
    if (bad && tid == 0) atomicCAS(a.info, 0, k0 + j + 1);
    __syncthreads();
    if (tid < j) S[tid * LDT + j] = S[tid * LDT + j] / d;
    if (tid == j) S[j * LDT + j] = d;
    __syncthreads();
    for (int i = ti; i < j; i += 16)
      for (int l = tl; l < j; l += 16) S[i * LDT + l] -= S[i * LDT + j] * S[l * LDT + j];
  }
  __syncthreads();
  // Wi = V^-1 (V = upper part of S), one column per thread by back substitution
  if (tid < NB) {
    const int c = tid;
    Wi[c * LDT + c] = 1.0 / S[c * LDT + c];
    for (int i = c - 1; i >= 0; --i) {
      double s = 0.0;
      for (int l = i + 1; l <= c; ++l) s = fma(S[i * LDT + l], Wi[l * LDT + c], s);
      Wi[i * LDT + c] = -s / S[i * LDT + i];
    }
  }
  __syncthreads();
  double* D = a.Dinv + (int64_t)a.kb * NB * NB;
  for (int idx = tid; idx < NB * NB; idx += 256) {
    const int r = idx >> 6, c = idx & 63;
    const double v = Wi[r * LDT + c];
    D[idx] = v;
    if (r < w && c < w && c >= r) a.F[(int64_t)(k0 + r) * a.ldf + k0 + c] = v;   // U_KK
  }
}

// ------------------------------------------------------------------ panel + row block
// blockIdx.x <  kb : row tile I = blockIdx.x,            V_IK = F_IK Winv^T   (in place)
// blockIdx.x >= kb : column tile J = blockIdx.x + 1,     U_KJ = Winv R_KJ     (in place)
__global__ __launch_bounds__(256) void panel_kernel(Sweep a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  double* As = reinterpret_cast<double*>(smem_raw);
  double* Bs = As + NB * LDT;
  const int k0 = a.kb * NB;
  const double* D = a.Dinv + (int64_t)a.kb * NB * NB;
  const bool is_panel = (int)blockIdx.x < a.kb;
  int r0, c0;
  if (is_panel) {
    r0 = blockIdx.x * NB; c0 = k0;
    stage_tile(As, a.F, a.ldf, r0, c0, a.n, a.n, false);          // A[i][l] = F[r0+i][k0+l]
    stage_tile(Bs, D, NB, 0, 0, NB, NB, false);                   // B[l][c] = Winv[c][l]
  } else {
    r0 = k0; c0 = (blockIdx.x + 1) * NB;
    stage_tile(As, D, NB, 0, 0, NB, NB, false);                   // A[r][l] = Winv[r][l]
    stage_tile(Bs, a.F, a.ldf, r0, c0, a.n, a.n, true);           // B[l][c] = F[k0+l][c0+c]
  }
  __syncthreads();
  double acc[4][4];
  mm64(As, Bs, acc);
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = r0 + 4 * ty + p, c = c0 + tx + 16 * q;
      if (r < a.n && c < a.n) a.F[(int64_t)r * a.ldf + c] = acc[p][q];
    }
}

// ----------------------------------------------------------------------------- update
// grid (nblk - 1, kb): blockIdx.y = row tile I (< K); column tile J = blockIdx.x, shifted past K.
//   J <  K : F_IJ -= V_IK V_JK^T   (only J >= I)
//   J >  K : F_IJ -= V_IK U_KJ
__global__ __launch_bounds__(256) void update_kernel(Sweep a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  double* As = reinterpret_cast<double*>(smem_raw);
  double* Bs = As + NB * LDT;
  const int I = blockIdx.y;
  int J = blockIdx.x;
  if (J >= a.kb) ++J;
  if (J < I) return;
  const int k0 = a.kb * NB, r0 = I * NB, c0 = J * NB;
  stage_tile(As, a.F, a.ldf, r0, k0, a.n, a.n, false);            // A[i][l] = V[r0+i][k0+l]
  if (J < a.kb) stage_tile(Bs, a.F, a.ldf, c0, k0, a.n, a.n, false);   // B[l][c] = V[c0+c][k0+l]
  else stage_tile(Bs, a.F, a.ldf, k0, c0, a.n, a.n, true);             // B[l][c] = U[k0+l][c0+c]
  __syncthreads();
  double acc[4][4];
  mm64(As, Bs, acc);
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = r0 + 4 * ty + p, c = c0 + tx + 16 * q;
      if (r < a.n && c < a.n) a.F[(int64_t)r * a.ldf + c] -= acc[p][q];
    }
}

// ------------------------------------------------------------------------------ close
// R_IK = -V_IK U_KK for every row tile I above K (in place over V_IK).
__global__ __launch_bounds__(256) void close_kernel(Sweep a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  double* As = reinterpret_cast<double*>(smem_raw);
  double* Bs = As + NB * LDT;
  const int k0 = a.kb * NB, r0 = blockIdx.x * NB;
  const double* D = a.Dinv + (int64_t)a.kb * NB * NB;
  stage_tile(As, a.F, a.ldf, r0, k0, a.n, a.n, false);
  stage_tile(Bs, D, NB, 0, 0, NB, NB, true);                      // B[l][c] = Winv[l][c]
  __syncthreads();
  double acc[4][4];
  mm64(As, Bs, acc);
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = r0 + 4 * ty + p, c = k0 + tx + 16 * q;
      if (r < a.n && c < a.n) a.F[(int64_t)r * a.ldf + c] = -acc[p][q];
    }
}

// --------------------------------------------------------------- extraction and splits
__device__ __forceinline__ uint16_t bf16_rne(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ float bf16_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// U (fp32, upper, zeros below) from F; its bf16 hi/lo split row-major (Uh, Ul) and
// transposed (Uth, Utl), all zero-padded to np x np.   grid (np/64, np/64), 256 threads.
__global__ __launch_bounds__(256) void extract_U_kernel(const double* F, int64_t ldf, int n, float* U, int64_t ldu,
                                                        uint16_t* Uh, uint16_t* Ul, uint16_t* Uth, uint16_t* Utl,
                                                        int64_t np) {
  __shared__ uint16_t th[64][66], tl[64][66];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int c = threadIdx.x & 63, rb = threadIdx.x >> 6;
  for (int p = 0; p < 16; ++p) {
    const int r = rb + 4 * p, gr = r0 + r, gc = c0 + c;
    float u = 0.f;
    if (gr < n && gc < n) {
      if (gc >= gr) u = (float)F[(int64_t)gr * ldf + gc];
      U[(int64_t)gr * ldu + gc] = u;
    }
    const uint16_t h = bf16_rne(u);
    const uint16_t l = bf16_rne(u - bf16_f32(h));
    Uh[(int64_t)gr * np + gc] = h;
    Ul[(int64_t)gr * np + gc] = l;
    th[r][c] = h;
    tl[r][c] = l;
  }
  __syncthreads();
  for (int p = 0; p < 16; ++p) {
    const int r = rb + 4 * p;            // r: column of U inside the tile, c: row of U
    Uth[(int64_t)(c0 + r) * np + r0 + c] = th[c][r];
    Utl[(int64_t)(c0 + r) * np + r0 + c] = tl[c][r];
  }
}

// bf16 hi/lo split of an fp32 matrix (rows flagged in `zero_rows` read as 0), padded to np x np.
__global__ __launch_bounds__(256) void split_rows_kernel(const float* A, int64_t lda, int n, const uint8_t* zero_rows,
                                                         uint16_t* Ah, uint16_t* Al, int64_t np) {
  const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x, r = blockIdx.y;
  if (c >= np) return;
  float v = 0.f;
  if (r < n && c < n && !(zero_rows && zero_rows[r])) v = A[r * lda + c];
  const uint16_t h = bf16_rne(v);
  Ah[r * np + c] = h;
  Al[r * np + c] = bf16_rne(v - bf16_f32(h));
}

}  // namespace gptaq

using namespace gptaq;

namespace {
struct PrepLayout {
  int64_t np;
  size_t off_F, off_Dinv, off_lam, off_dead, off_O, off_b[6], total;
};
PrepLayout prep_layout(int64_t n) {
  PrepLayout L;
  const int tile = gemm_tile_for(n, n);
  L.np = round_up(n, tile);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += (bytes + 255) / 256 * 256; return r; };
  L.off_lam = take(256);
  L.off_F = take((size_t)n * n * 8);
  L.off_Dinv = take((size_t)round_up(n, NB) * NB * 8);
  L.off_dead = take((size_t)n);
  L.off_O = take((size_t)L.np * L.np * 4);
  for (int i = 0; i < 6; ++i) L.off_b[i] = take((size_t)L.np * L.np * 2);
  L.total = o;
  return L;
}
bool g_prep_attr = false;
}  // namespace

extern "C" size_t gptaq_prepare_workspace_bytes(int64_t n) {
  if (n <= 0) return 0;
  return prep_layout(n).total;
}

extern "C" int gptaq_prepare(float* H, float* dXXT, int64_t n, int64_t ldh, float damp, uint8_t* dead,
                             int32_t* info, void* ws, size_t ws_bytes, void* stream) {
  if (!H || !dXXT || !info || !ws) return GPTAQ_ENULL;
  if (n <= 0 || ldh < n || n > 65535 * NB / 2 || !(damp >= 0.f)) return GPTAQ_EDIM;
  if ((uintptr_t)ws & 255) return GPTAQ_EWORKSPACE;
  const PrepLayout L = prep_layout(n);
  if (ws_bytes < L.total) return GPTAQ_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  if (!g_prep_attr) {
    const void* fns[4] = {(const void*)&diag_kernel, (const void*)&panel_kernel, (const void*)&update_kernel,
                          (const void*)&close_kernel};
    for (const void* f : fns) {
      hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, MM_LDS);
      if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
    }
    g_prep_attr = true;
  }
  unsigned char* base = (unsigned char*)ws;
  double* lam = (double*)(base + L.off_lam);
  double* F = (double*)(base + L.off_F);
  double* Dinv = (double*)(base + L.off_Dinv);
  uint8_t* deadbuf = dead ? dead : (uint8_t*)(base + L.off_dead);
  float* Obuf = (float*)(base + L.off_O);
  uint16_t* bb[6];
  for (int i = 0; i < 6; ++i) bb[i] = (uint16_t*)(base + L.off_b[i]);
  const int ni = (int)n;

  hipLaunchKernelGGL(diag_stats_kernel, dim3(1), dim3(1024), 0, s, H, ldh, ni, damp, deadbuf, lam, info);
  GPTAQ_LAUNCH_CHECK();
  hipLaunchKernelGGL(build_F_kernel, dim3((unsigned)((n + 255) / 256), (unsigned)n), dim3(256), 0, s, H, ldh, ni,
                     lam, F, n);
  GPTAQ_LAUNCH_CHECK();

  {
  ProfScope sweep_scope(kProfFactor, s);
  Sweep a;
  a.F = F; a.ldf = n; a.n = ni; a.nblk = (int)((n + NB - 1) / NB); a.Dinv = Dinv; a.info = info;
  for (int kb = a.nblk - 1; kb >= 0; --kb) {
    a.kb = kb;
    hipLaunchKernelGGL(diag_kernel, dim3(1), dim3(256), MM_LDS, s, a);
    GPTAQ_LAUNCH_CHECK();
    if (a.nblk > 1) {
      hipLaunchKernelGGL(panel_kernel, dim3(a.nblk - 1), dim3(256), MM_LDS, s, a);
      GPTAQ_LAUNCH_CHECK();
    }
    if (kb > 0) {
      if (a.nblk > 1) {
        hipLaunchKernelGGL(update_kernel, dim3(a.nblk - 1, kb), dim3(256), MM_LDS, s, a);
        GPTAQ_LAUNCH_CHECK();
      }
      hipLaunchKernelGGL(close_kernel, dim3(kb), dim3(256), MM_LDS, s, a);
      GPTAQ_LAUNCH_CHECK();
    }
  }

  }
  // U -> H (fp32) and the bf16 splits; dXXT (dead rows zeroed) split.
  const int64_t np = L.np;
  uint16_t *Uh = bb[0], *Ul = bb[1], *Uth = bb[2], *Utl = bb[3], *Ah = bb[4], *Al = bb[5];
  hipLaunchKernelGGL(extract_U_kernel, dim3((unsigned)(np / 64), (unsigned)(np / 64)), dim3(256), 0, s, F, n, ni, H,
                     ldh, Uh, Ul, Uth, Utl, np);
  GPTAQ_LAUNCH_CHECK();
  hipLaunchKernelGGL(split_rows_kernel, dim3((unsigned)((np + 255) / 256), (unsigned)np), dim3(256), 0, s, dXXT, ldh,
                     ni, deadbuf, Ah, Al, np);
  GPTAQ_LAUNCH_CHECK();

  const int tile = gemm_tile_for(n, n);
  GemmBatch b;
  b.nprob = 1; b.tile = tile;
  GemmProblem& g = b.p[0];
  // O = triu(dXXT U^T, 1): O[i][a] = sum_{b >= a} dXXT[i][b] U[a][b]
  g.C = Obuf; g.ldc = np; g.M = ni; g.N = ni; g.K = (int)np;
  g.tiles_m = g.tiles_n = (int)(np / tile);
  g.kind = 2; g.nterm = 1; g.tile_mode = 1; g.k_mode = 1; g.store_mode = 2;
  g.term[0] = {{Ah, Al}, {Uh, Ul}, np, np, 32, 32};
  hipError_t e;
  {
    ProfScope ps(kProfPGemm, s);
    e = launch_gemm(b, s);
  }
  if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
  // split O (reuses the dXXT split buffers), then P = O U: P[i][j] = sum_{i < a <= j} O[i][a] U[a][j]
  hipLaunchKernelGGL(split_rows_kernel, dim3((unsigned)((np + 255) / 256), (unsigned)np), dim3(256), 0, s, Obuf, np,
                     ni, (const uint8_t*)nullptr, Ah, Al, np);
  GPTAQ_LAUNCH_CHECK();
  g.C = dXXT; g.ldc = ldh; g.k_mode = 2;
  g.term[0] = {{Ah, Al}, {Uth, Utl}, np, np, 32, 32};
  {
    ProfScope ps(kProfPGemm, s);
    e = launch_gemm(b, s);
  }
  if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
  return GPTAQ_OK;
}
