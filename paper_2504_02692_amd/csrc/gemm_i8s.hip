// fp64-grade rank-k products on the int8 matrix cores of gfx950 (digit-sliced integer arithmetic).
//
// The factorisation of the damped Hessian and the inversion of its factor (Algorithm 1, line 3) are a
// sweep of rank-256 updates  C = beta C + alpha A B^T  on fp64 data.  The fp64 matrix rate of this chip is
// far below its int8 rate, so the operands are rewritten as fixed-point numbers with a power-of-two scale
// per row and six signed 8-bit digits,
//     a[r][k] ~ 2^(E_r - 46) * sum_i d_i[r][k] 256^(5-i),     d_0 in [-64, 64], d_1..5 in [-128, 127],
// and the product becomes 21 exact int8 x int8 -> int32 products (the digit pairs with i + j <= 5; the
// dropped pairs lie below 2^-46 of max|a_r| max|b_c| K).  Pairs of equal weight i + j share an int32
// accumulator (at most 6 * 256 * 2^14 < 2^31), and the six accumulators are combined in fp64 at the end.
// The result carries an absolute error of about 2^-44 max_k|a| max_k|b| per term of the dot product: a
// normwise bound of the same kind as a floating-point product's, ~2^7 coarser than native fp64 and far
// below what the fp32 outputs of the solve resolve.
//
// Layout of a sliced operand (written by slice_i8_kernel, consumed by gemm_i8s_kernel): digit plane i,
// k-chunk c (32 digits), row slab (32 rows) form one 1 KB block, stored in exactly the order the block has
// in LDS, so a wavefront moves it with one global -> LDS load of 16 bytes per lane.  Inside the block, row
// r and 16-byte half h sit at 256 (r / 8) + 16 (2 (r % 8) + (h ^ ((r / 8) & 1))): the 16 rows that one
// clock of a ds_read_b128 serves fall into 16 different 16-byte slots of a 256-byte LDS line pair.
#include "common.h"

namespace gptaq {

typedef int __attribute__((ext_vector_type(4))) i32x4;
typedef int __attribute__((ext_vector_type(16))) i32x16;

namespace {
constexpr int NP = kI8Planes;                // digit planes
constexpr int BM = 128, BN = 64;             // workgroup tile: four wavefronts 2 x 2, each 64 x 32
constexpr int KC = 32;                       // digits per k-chunk = one MFMA k-step
constexpr int SLABS_A = BM / 32, SLABS_B = BN / 32;
constexpr int STAGE = NP * (BM + BN) * KC;   // 36 KB: all planes of both operands for one k-chunk
constexpr int NSTAGE = 3;
constexpr int LOADS = NP * (SLABS_A + SLABS_B);   // 1 KB wave loads per chunk
constexpr int LPW = LOADS / 4;                    // per wavefront
static_assert(LOADS % 4 == 0, "loads divide over the four wavefronts");

__device__ __forceinline__ void wg_barrier_nofence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
template <int N> __device__ __forceinline__ void wait_vm_lds() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4));     // vmcnt <= N, lgkmcnt == 0
}
}  // namespace

// ---------------------------------------------------------------------------------------------- slicing
// Source element (r, k), r < R, k < K <= 256, at src[r * sr + k * sk]; one of the strides is 1.
// One workgroup slices one slab of 32 rows: thread t owns 32 consecutive k of one row (one k-chunk).
// Rows >= R of the last slab and k >= K are written as zeros; slabs past the last row are left alone (a
// product only stores the rows it was asked for, whatever digits the padding holds).
__global__ __launch_bounds__(256) void slice_i8_kernel(const double* src, int64_t sr, int64_t sk, int R, int K,
                                                       uint8_t* planes, int64_t plane_stride, int64_t chunk_stride,
                                                       double* scale) {
  __shared__ double smax[32][9];
  const int t = threadIdx.x;
  const bool kmajor = sr == 1;                   // consecutive threads along the contiguous direction
  const int rl = kmajor ? (t & 31) : (t >> 3), c = kmajor ? (t >> 5) : (t & 7);
  const int r = blockIdx.x * 32 + rl;
  double v[KC];
  double mx = 0.0;
#pragma unroll
  for (int q = 0; q < KC; ++q) {
    const int k = c * KC + q;
    v[q] = (r < R && k < K) ? src[(int64_t)r * sr + (int64_t)k * sk] : 0.0;
    mx = fmax(mx, fabs(v[q]));
  }
  smax[rl][c] = mx;
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 8; ++q) mx = fmax(mx, smax[rl][q]);
  int e = 0;
  if (mx > 0.0) (void)frexp(mx, &e);              // mx = f * 2^e, f in [0.5, 1)
  if (c == 0) scale[r] = ldexp(1.0, e - 26);      // the product of two scales carries 2^-52: see the epilogue
  uint32_t w[NP][8];
#pragma unroll
  for (int i = 0; i < NP; ++i)
#pragma unroll
    for (int q = 0; q < 8; ++q) w[i][q] = 0;
#pragma unroll
  for (int q = 0; q < KC; ++q) {
    long long n = (long long)rint(ldexp(v[q], 46 - e));        // |n| <= 2^46
#pragma unroll
    for (int i = NP - 1; i >= 1; --i) {
      const int d = (int)((n + 128) & 255) - 128;              // digit in [-128, 127], n - d divisible by 256
      n = (n - d) >> 8;
      w[i][q >> 2] |= (uint32_t)(d & 255) << (8 * (q & 3));
    }
    w[0][q >> 2] |= (uint32_t)((int)n & 255) << (8 * (q & 3));
  }
  const int line = rl >> 3;
  uint8_t* blk = planes + (int64_t)c * chunk_stride + (int64_t)blockIdx.x * 1024 + line * 256;
#pragma unroll
  for (int i = 0; i < NP; ++i)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int slot = ((rl & 7) << 1) | (h ^ (line & 1));
      *reinterpret_cast<u32x4*>(blk + (int64_t)i * plane_stride + slot * 16) =
          u32x4{w[i][4 * h], w[i][4 * h + 1], w[i][4 * h + 2], w[i][4 * h + 3]};
    }
}

// ------------------------------------------------------------------------------------------------ product
__global__ __launch_bounds__(256) void gemm_i8s_kernel(I8Gemm g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // ---- which tile.  Workgroups go round-robin to the 8 XCDs; each XCD gets one contiguous run of the tile
  // list, and the list runs through groups of four tile rows column by column, so the tiles an XCD works on
  // at one time form a 4 x 8 patch whose operand slabs (1.5 MB) stay in that XCD's L2.
  int id = blockIdx.x;
  {
    const int ntile = gridDim.x, per = ntile >> 3, rem = ntile & 7, xcd = id & 7, loc = id >> 3;
    id = xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
  }
  int tm, tn;
  {
    // with upper_only, a group of tile rows starts at the tile column of its first row's diagonal
    int first = 0, gsz, c0, cnt;
    for (;;) {
      gsz = min(4, g.tiles_m - first);
      c0 = g.upper_only ? min(first * (BM / BN), g.tiles_n) : 0;
      cnt = gsz * (g.tiles_n - c0);
      if (id < cnt || first + gsz >= g.tiles_m) break;
      id -= cnt;
      first += gsz;
    }
    if (id >= cnt) return;                     // (cannot happen: the grid is the sum of the group counts)
    tm = first + id % gsz;
    tn = c0 + id / gsz;
  }
  const int i0 = tm * BM, j0 = tn * BN;
  if (g.upper_only && j0 + BN <= i0) return;

  // loads: block q of a chunk (q < NP * SLABS_A: plane q / SLABS_A, slab q % SLABS_A of A; then B) goes to
  // stage + 1024 q.  Wavefront w moves blocks w * LPW .. w * LPW + LPW - 1.
  auto load_chunk = [&](int c, int stage) {
#pragma unroll
    for (int u = 0; u < LPW; ++u) {
      const int q = wave * LPW + u;
      const uint8_t* src;
      if (q < NP * SLABS_A)
        src = g.A + (int64_t)(q / SLABS_A) * g.a_plane + (int64_t)c * g.a_chunk + (int64_t)(i0 + (q % SLABS_A) * 32) * KC;
      else
        src = g.B + (int64_t)((q - NP * SLABS_A) / SLABS_B) * g.b_plane + (int64_t)c * g.b_chunk +
              (int64_t)(j0 + ((q - NP * SLABS_A) % SLABS_B) * 32) * KC;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + lane * 16),
                                       (__attribute__((address_space(3))) void*)(smem + stage * STAGE + q * 1024), 16, 0, 0);
    }
  };

  i32x16 acc[NP][2];
#pragma unroll
  for (int s = 0; s < NP; ++s)
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[s][f][v] = 0;

  const int rl = lane & 31, line = rl >> 3;
  const int lane_off = line * 256 + ((((rl & 7) << 1) | ((lane >> 5) ^ (line & 1))) << 4);
  const int a_off = wm * 2 * 1024 + lane_off, b_off = NP * SLABS_A * 1024 + wn * 1024 + lane_off;

  const int nch = g.nchunk;
  load_chunk(0, 0);
  if (nch > 1) load_chunk(1, 1);
  for (int c = 0; c < nch; ++c) {
    // loads return in order: "at most LPW outstanding" means chunk c has landed (its successor may not have)
    if (c + 1 < nch) wait_vm_lds<LPW>(); else wait_vm_lds<0>();
    wg_barrier_nofence();                          // chunk c visible to all; every wave is done with chunk c - 1
    if (c + 2 < nch) load_chunk(c + 2, (c + 2) % NSTAGE);
    const unsigned char* st = smem + (c % NSTAGE) * STAGE;
    i32x4 a[NP][2], b[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      b[p] = *reinterpret_cast<const i32x4*>(st + b_off + p * SLABS_B * 1024);
#pragma unroll
      for (int f = 0; f < 2; ++f) a[p][f] = *reinterpret_cast<const i32x4*>(st + a_off + (p * SLABS_A + f) * 1024);
    }
    // digit pair (i, j) adds into the accumulator of weight i + j; consecutive MFMAs use different accumulators
#pragma unroll
    for (int i = 0; i < NP; ++i)
#pragma unroll
      for (int j = 0; j + i < NP; ++j)
#pragma unroll
        for (int f = 0; f < 2; ++f)
          acc[i + j][f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][f], b[j], acc[i + j][f], 0, 0, 0);
  }

  // ---- epilogue.  a b = 2^(Ea + Eb - 92) sum_s acc_s 256^(10 - s) = 2^(Ea + Eb - 52) t with
  // t = sum_s acc_s 256^(5 - s) (Horner form below), and the row scales are 2^(E - 26): value = sa sb t.
  // 32x32 result block: register v of a lane holds row 8 (v / 4) + 4 (lane / 32) + v % 4, column lane % 32.
  const int col = j0 + wn * 32 + rl;
  const double sbv = g.alpha * g.sb[col];          // scale arrays are padded to whole tiles
#pragma unroll
  for (int f = 0; f < 2; ++f) {
    const int rbase = i0 + wm * 64 + f * 32 + 4 * (lane >> 5);
    double old[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = rbase + 8 * (v >> 2) + (v & 3);
      old[v] = (g.beta && row < g.M && col < g.N) ? g.C[(int64_t)row * g.ldc + col] : 0.0;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = rbase + 8 * (v >> 2) + (v & 3);
      double t = (double)acc[0][f][v];
#pragma unroll
      for (int s = 1; s < NP; ++s) t = fma(t, 256.0, (double)acc[s][f][v]);
      if (row < g.M && col < g.N) g.C[(int64_t)row * g.ldc + col] = fma(g.sa[row] * sbv, t, old[v]);
    }
  }
}

static bool g_i8_attr = false;

hipError_t launch_slice_i8(const double* src, int64_t sr, int64_t sk, int R, int K, const I8Operand& o, hipStream_t s) {
  if (R <= 0) return hipSuccess;
  if (K > kI8MaxK || (sr != 1 && sk != 1) || R > o.rows_pad) return hipErrorInvalidValue;
  hipLaunchKernelGGL(slice_i8_kernel, dim3((unsigned)((R + 31) / 32)), dim3(256), 0, s, src, sr, sk, R, K, o.planes,
                     o.plane_stride(), o.chunk_stride(), o.scale);
  return hipGetLastError();
}

hipError_t launch_gemm_i8s(const I8Operand& A, int a_row0, const I8Operand& B, int b_row0, double* C, int64_t ldc, int M,
                           int N, int K, double alpha, int beta, int upper_only, hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
  if (K > kI8MaxK || (a_row0 % BM) || (b_row0 % BN)) return hipErrorInvalidValue;
  I8Gemm g;
  g.tiles_m = (M + BM - 1) / BM;
  g.tiles_n = (N + BN - 1) / BN;
  if (a_row0 + g.tiles_m * BM > A.rows_pad || b_row0 + g.tiles_n * BN > B.rows_pad) return hipErrorInvalidValue;
  if (!g_i8_attr) {
    hipError_t e = hipFuncSetAttribute((const void*)&gemm_i8s_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       NSTAGE * STAGE);
    if (e != hipSuccess) return e;
    g_i8_attr = true;
  }
  g.A = A.planes + (int64_t)a_row0 * KC; g.a_plane = A.plane_stride(); g.a_chunk = A.chunk_stride(); g.sa = A.scale + a_row0;
  g.B = B.planes + (int64_t)b_row0 * KC; g.b_plane = B.plane_stride(); g.b_chunk = B.chunk_stride(); g.sb = B.scale + b_row0;
  g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.nchunk = (K + KC - 1) / KC; g.beta = beta; g.upper_only = upper_only;
  g.alpha = alpha;
  int total = 0;
  for (int first = 0; first < g.tiles_m; first += 4) {
    const int gsz = g.tiles_m - first < 4 ? g.tiles_m - first : 4;
    const int c0 = upper_only ? (first * (BM / BN) < g.tiles_n ? first * (BM / BN) : g.tiles_n) : 0;
    total += gsz * (g.tiles_n - c0);
  }
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(gemm_i8s_kernel, dim3((unsigned)total), dim3(256), NSTAGE * STAGE, s, g);
  return hipGetLastError();
}

}  // namespace gptaq
