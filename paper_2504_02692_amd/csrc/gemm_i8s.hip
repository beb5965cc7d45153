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
constexpr int BN = 64;                       // tile columns
constexpr int KC = 32;                       // digits per k-chunk = one MFMA k-step
constexpr int SLABS_B = BN / 32;
// Two shapes.  BM = 128: one workgroup per CU, four wavefronts 2 x 2, each 64 x 32, a ring of four chunks.
// BM = 64: two workgroups per CU (half the registers and LDS each), wavefronts 32 x 32, a ring of three: the
// stalls and the epilogue of one workgroup run under the MFMAs of the other.
template <int BM> struct Shape {
  static constexpr int SLABS_A = BM / 32, FRM = BM / 64;
  static constexpr int STAGE = NP * (BM + BN) * KC;         // all planes of both operands for one k-chunk
  static constexpr int NSTAGE = BM == 128 ? 4 : 3, AHEAD = NSTAGE - 1;
  static constexpr int LOADS = NP * (SLABS_A + SLABS_B);    // 1 KB wave loads per chunk
  static constexpr int LPW = LOADS / 4;                     // per wavefront
  static constexpr int NM = (NP * (NP + 1) / 2) * FRM;      // MFMAs per chunk and wavefront
  static constexpr int EPI = 16 * FRM + 4 * FRM + 1;        // old C, row exponents (four rows per load), column exponent
  static_assert(LOADS % 4 == 0 && (AHEAD - 1) * LPW + EPI <= 63, "loads divide over the wavefronts; vmcnt has 6 bits");
};

__device__ __forceinline__ void wg_barrier_nofence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
template <int N> __device__ __forceinline__ void wait_vm_lds() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4));     // vmcnt <= N, lgkmcnt == 0
}
// the same for a count known at run time: `chunks` later chunks of LPW loads, plus the epilogue's EPI loads
template <int LPW, int EPI> __device__ __forceinline__ void wait_vm_lds_for(int chunks, bool epi) {
  if (epi) {
    if (chunks >= 2) wait_vm_lds<2 * LPW + EPI>(); else if (chunks == 1) wait_vm_lds<LPW + EPI>(); else wait_vm_lds<EPI>();
  } else {
    if (chunks >= 2) wait_vm_lds<2 * LPW>(); else if (chunks == 1) wait_vm_lds<LPW>(); else wait_vm_lds<0>();
  }
}
}  // namespace

// ---------------------------------------------------------------------------------------------- slicing
// Source element (r, k), r < R, k < K <= 256, at src[r * sr + k * sk]; one of the strides is 1.
// One workgroup slices one slab of 32 rows: thread t owns 32 consecutive k of one row (one k-chunk).
// Rows >= R of the last slab and k >= K are written as zeros; slabs past the last row are left alone (a
// product only stores the rows it was asked for, whatever digits the padding holds).
__global__ __launch_bounds__(256) void slice_i8_kernel(const double* src, int64_t sr, int64_t sk, int R, int K,
                                                       uint8_t* planes, int64_t plane_stride, int64_t chunk_stride,
                                                       int32_t* scale) {
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
  if (c == 0) scale[r] = e - 26;                  // the product of two scaled rows carries 2^-52: see the epilogue
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
// Each workgroup walks its share of the tile list (one tile, or many for large products), and the k-chunks of
// consecutive tiles form one stream through the LDS ring, so the first chunks of the next tile arrive while the current one is
// finished and written out.
template <int BM>
__global__ __launch_bounds__(256, BM == 128 ? 1 : 2) void gemm_i8s_kernel(I8Gemm g) {
  using S = Shape<BM>;
  constexpr int SLABS_A = S::SLABS_A, FRM = S::FRM, STAGE = S::STAGE, NSTAGE = S::NSTAGE, AHEAD = S::AHEAD, LPW = S::LPW;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // ---- which tiles.  Workgroups go round-robin to the 8 XCDs; each XCD gets one contiguous run of the tile
  // list and its workgroups take the tiles of that run in turn.  The list runs through groups of four tile
  // rows column by column, so the tiles an XCD works on at one time form a 4 x 8 patch whose operand slabs
  // (1.5 MB) stay in that XCD's L2.
  int t_next, t_end, t_step;
  {
    const int nwg = gridDim.x, xcd = blockIdx.x & 7, loc = blockIdx.x >> 3;
    const int per = g.ntile >> 3, rem = g.ntile & 7;
    t_next = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + loc;
    t_end = t_next - loc + per + (xcd < rem ? 1 : 0);
    t_step = (nwg >> 3) + (xcd < (nwg & 7) ? 1 : 0);
  }
  struct Tile { int i0, j0; bool ok; };
  // the next tile of this workgroup that has work (with upper_only, a group of tile rows starts at the tile
  // column of its first row's diagonal, and the few tiles of its other rows left of theirs are skipped)
  auto advance = [&]() -> Tile {
    while (t_next < t_end) {
      int id = t_next;
      t_next += t_step;
      int first = 0, gsz, c0, cnt;
      for (;;) {
        gsz = min(4, g.tiles_m - first);
        c0 = g.upper_only ? min(first * (BM / BN), g.tiles_n) : 0;
        cnt = gsz * (g.tiles_n - c0);
        if (id < cnt || first + gsz >= g.tiles_m) break;
        id -= cnt;
        first += gsz;
      }
      if (id >= cnt) continue;
      const int i0 = (first + id % gsz) * BM, j0 = (c0 + id / gsz) * BN;
      if (g.upper_only && j0 + BN <= i0) continue;
      return Tile{i0, j0, true};
    }
    return Tile{0, 0, false};
  };

  // loads: a chunk is NP * SLABS_A blocks of A (plane p, slab f at stage + 1024 (SLABS_A p + f)) and then
  // NP * SLABS_B blocks of B.  BM = 128: wavefront w moves slab w of every A plane and B blocks 3 w .. 3 w + 2;
  // BM = 64: wavefronts 0, 1 move the A blocks 6 w .. 6 w + 5, wavefronts 2, 3 the B blocks.  One load at a time
  // between the MFMAs of the chunk being multiplied (a wave stalls some tens of clocks per load it hands to the
  // memory pipeline; in a burst that is time the matrix unit idles).
  static_assert((BM == 128 && LPW == NP + 3) || (BM == 64 && LPW == NP), "load assignment");
  int lstage = 0;                                // ring position of the next chunk to load
  struct LoadCtx { const uint8_t* pa; const uint8_t* pb; unsigned char* st; bool on; };
  auto begin_load = [&](const Tile& t, int c, bool on) {
    LoadCtx L;
    L.on = on;
    L.st = smem + lstage * STAGE;
    L.pa = g.A + (int64_t)c * g.a_chunk + (int64_t)t.i0 * KC + lane * 16;
    L.pb = g.B + (int64_t)c * g.b_chunk + (int64_t)t.j0 * KC + lane * 16;
    if (on) lstage = lstage == NSTAGE - 1 ? 0 : lstage + 1;
    return L;
  };
  auto load_a = [&](const LoadCtx& L, int q) {   // A block q = SLABS_A * plane + slab
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(L.pa + (q / SLABS_A) * g.a_plane + (q % SLABS_A) * 1024),
                                     (__attribute__((address_space(3))) void*)(L.st + q * 1024), 16, 0, 0);
  };
  auto load_b = [&](const LoadCtx& L, int q) {   // B block q = SLABS_B * plane + slab
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(L.pb + (q / SLABS_B) * g.b_plane + (q % SLABS_B) * 1024),
                                     (__attribute__((address_space(3))) void*)(L.st + (NP * SLABS_A + q) * 1024), 16, 0, 0);
  };
  auto load_one = [&](const LoadCtx& L, int u) {
    if (!L.on) return;
    if constexpr (BM == 128) {
      if (u < NP) load_a(L, u * SLABS_A + wave); else load_b(L, wave * 3 + (u - NP));
    } else {
      if (wave < 2) load_a(L, wave * LPW + u); else load_b(L, (wave - 2) * LPW + u);
    }
  };

  const int rl = lane & 31, line = rl >> 3;
  const int lane_off = line * 256 + ((((rl & 7) << 1) | ((lane >> 5) ^ (line & 1))) << 4);
  const int a_off = wm * FRM * 1024 + lane_off, b_off = NP * SLABS_A * 1024 + wn * 1024 + lane_off;
  const int nch = g.nchunk;                      // >= AHEAD: the chunks in flight never reach past the next tile

  Tile cur = advance();
  if (!cur.ok) return;
  Tile nxt = advance();
#pragma unroll
  for (int c = 0; c < AHEAD; ++c) {
    const LoadCtx L0 = begin_load(cur, c, true);
#pragma unroll
    for (int u = 0; u < LPW; ++u) load_one(L0, u);
  }
  int cstage = 0;                                // ring position of the next chunk to multiply
  bool first = true;
  constexpr int EPI_LOADS = S::EPI;
  for (;;) {
    i32x16 acc[NP][FRM];
#pragma unroll
    for (int s = 0; s < NP; ++s)
#pragma unroll
      for (int f = 0; f < FRM; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][f][v] = 0;
    // 32x32 result block: register v of a lane holds row 8 (v / 4) + 4 (lane / 32) + v % 4, column lane % 32.
    const int col = cur.j0 + wn * 32 + rl;
    const int rbase = cur.i0 + wm * (32 * FRM) + 4 * (lane >> 5);
    double old[FRM][16];
    i32x4 ea[FRM][4];
    int eb;

    for (int c = 0; c < nch; ++c) {
      // This wave's loads return in order, so "at most N outstanding" means that everything issued before
      // the last N has landed; N counts what was issued after the chunk needed now: the chunks up to AHEAD - 1
      // further on and, in the first tile, the epilogue's loads (issued right after the first AHEAD chunks).
      // Stores of the previous epilogue may still be counted: that only makes the wait longer.  The first
      // AHEAD chunks of a later tile were waited for before that epilogue.
      int later = 0;
#pragma unroll
      for (int d = 1; d < AHEAD; ++d) later += (c + d < nch || nxt.ok) ? 1 : 0;
      if (c >= AHEAD || (first && c == 0)) wait_vm_lds_for<LPW, EPI_LOADS>(later, false);
      else if (first) wait_vm_lds_for<LPW, EPI_LOADS>(later, true);
      else wait_vm_lds<63>();
      wg_barrier_nofence();                        // this chunk is visible to all; every wave is done with the one before
      if (c == 0) {
        // What the epilogue needs from memory is requested now and arrives while the tile is multiplied.
        // The addresses are clamped instead of predicated: the number of loads issued must not depend on data.
        const int cc = min(col, g.N - 1);
#pragma unroll
        for (int f = 0; f < FRM; ++f)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = min(rbase + f * 32 + 8 * (v >> 2) + (v & 3), g.M - 1);
            old[f][v] = g.C[(int64_t)row * g.ldc + cc];
          }
#pragma unroll
        for (int f = 0; f < FRM; ++f)
#pragma unroll
          for (int q = 0; q < 4; ++q) ea[f][q] = *reinterpret_cast<const i32x4*>(g.sa + rbase + f * 32 + 8 * q);
        eb = g.sb[col];
      }
      const bool in_tile = c + AHEAD < nch;
      const LoadCtx L = begin_load(in_tile ? cur : nxt, in_tile ? c + AHEAD : c + AHEAD - nch, in_tile || nxt.ok);
      const unsigned char* st = smem + cstage * STAGE;
      cstage = cstage == NSTAGE - 1 ? 0 : cstage + 1;
      // Fragments are read in the order in which the MFMAs first need them (LDS returns in order, so the
      // first MFMA waits for three reads only, and the rest arrive behind running MFMAs): the digit pairs
      // (i, j) are taken by max(i, j), so plane p of A and of B comes into play at step p.
      // (In two batches: the LDS counter of a wave holds 15 outstanding reads, and with more than that in
      // flight the compiler waits for all of them at once.)
      i32x4 a[NP][FRM], b[NP];
      auto read_plane = [&](int p) {
#pragma unroll
        for (int f = 0; f < FRM; ++f) a[p][f] = *reinterpret_cast<const i32x4*>(st + a_off + (p * SLABS_A + f) * 1024);
        b[p] = *reinterpret_cast<const i32x4*>(st + b_off + p * SLABS_B * 1024);
      };
#pragma unroll
      for (int p = 0; p < NP / 2; ++p) read_plane(p);
      __builtin_amdgcn_sched_barrier(0);
      // pair (i, j) adds into the accumulator of weight i + j; an accumulator is never used by two MFMAs in a row
      int m = 0;
      auto pair = [&](int i, int j) {
#pragma unroll
        for (int f = 0; f < FRM; ++f) {
          acc[i + j][f] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i][f], b[j], acc[i + j][f], 0, 0, 0);
          if (m == 2) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = NP / 2; p < NP; ++p) read_plane(p);
            __builtin_amdgcn_sched_barrier(0);
          }
          constexpr int GAP = S::NM / LPW;             // MFMAs between two loads
          if (m % GAP == 1 && m / GAP < LPW) {
            __builtin_amdgcn_sched_barrier(0);
            load_one(L, m / GAP);
            __builtin_amdgcn_sched_barrier(0);
          }
          ++m;
        }
      };
#pragma unroll
      for (int p = 0; p < NP; ++p) {
#pragma unroll
        for (int q = 0; q < p; ++q)
          if (p + q < NP) { pair(q, p); pair(p, q); }
        if (2 * p < NP) pair(p, p);
      }
    }

    // ---- epilogue.  a b = 2^(Ea + Eb - 92) sum_s acc_s 256^(10 - s) = 2^(Ea + Eb - 52) t with
    // t = sum_s acc_s 256^(5 - s) (Horner form below); the stored row exponents are E - 26.
    wait_vm_lds<0>();                                // old C and exponents; the next tile's first three chunks
#pragma unroll
    for (int f = 0; f < FRM; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = rbase + f * 32 + 8 * (v >> 2) + (v & 3);
        double t = (double)acc[0][f][v];
#pragma unroll
        for (int s = 1; s < NP; ++s) t = fma(t, 256.0, (double)acc[s][f][v]);
        t = ldexp(t, ea[f][v >> 2][v & 3] + eb);
        if (row < g.M && col < g.N) g.C[(int64_t)row * g.ldc + col] = g.beta ? fma(g.alpha, t, old[f][v]) : g.alpha * t;
      }
    if (!nxt.ok) break;
    first = false;
    cur = nxt;
    nxt = advance();
  }
}

hipError_t launch_slice_i8(const double* src, int64_t sr, int64_t sk, int R, int K, const I8Operand& o, hipStream_t s) {
  if (R <= 0) return hipSuccess;
  if (K > kI8MaxK || (sr != 1 && sk != 1) || R > o.rows_pad) return hipErrorInvalidValue;
  hipLaunchKernelGGL(slice_i8_kernel, dim3((unsigned)((R + 31) / 32)), dim3(256), 0, s, src, sr, sk, R, K, o.planes,
                     o.plane_stride(), o.chunk_stride(), o.scale);
  return hipGetLastError();
}

// Workgroups per launch, at most (for BM = 128; twice as many of the half-size ones).  A workgroup fills a CU or
// half of one, and the products run beside the small sequential kernels of the other chain of the sweep, which
// can only start on a CU that a workgroup has left: with one workgroup per CU for the whole launch those kernels
// waited (n = 11008: 32.6 ms per prepare; 31.5 with 512, 30.7 with 1024, 30.6 with one tile per workgroup).  1024
// keeps the workgroups of the sweep's products short and still lets very large products (n >= 28672) run tens of
// tiles per workgroup.
constexpr int kI8Workgroups = 1024;

template <int BM>
static hipError_t launch_shape(const I8Operand& A, int a_row0, const I8Operand& B, int b_row0, double* C, int64_t ldc, int M,
                               int N, int K, double alpha, int beta, int upper_only, hipStream_t s) {
  using S = Shape<BM>;
  static LdsLimitOnce lds_once;                  // per instantiation
  I8Gemm g;
  g.tiles_m = (M + BM - 1) / BM;
  g.tiles_n = (N + BN - 1) / BN;
  if (a_row0 + g.tiles_m * BM > A.rows_pad || b_row0 + g.tiles_n * BN > B.rows_pad) return hipErrorInvalidValue;
  {
    const hipError_t e = lds_once.ensure((const void*)&gemm_i8s_kernel<BM>, S::NSTAGE * S::STAGE);
    if (e != hipSuccess) return e;
  }
  g.A = A.planes + (int64_t)a_row0 * KC; g.a_plane = A.plane_stride(); g.a_chunk = A.chunk_stride(); g.sa = A.scale + a_row0;
  g.B = B.planes + (int64_t)b_row0 * KC; g.b_plane = B.plane_stride(); g.b_chunk = B.chunk_stride(); g.sb = B.scale + b_row0;
  g.C = C; g.ldc = ldc; g.M = M; g.N = N; g.beta = beta; g.upper_only = upper_only;
  const int nch = (K + KC - 1) / KC;               // (a sliced operand is zero past its K)
  g.nchunk = nch < S::AHEAD ? S::AHEAD : nch;
  g.alpha = alpha;
  int total = 0;
  for (int first = 0; first < g.tiles_m; first += 4) {
    const int gsz = g.tiles_m - first < 4 ? g.tiles_m - first : 4;
    const int c0 = upper_only ? (first * (BM / BN) < g.tiles_n ? first * (BM / BN) : g.tiles_n) : 0;
    total += gsz * (g.tiles_n - c0);
  }
  if (total == 0) return hipSuccess;
  g.ntile = total;
  const int cap = kI8Workgroups * (128 / BM);
  hipLaunchKernelGGL(gemm_i8s_kernel<BM>, dim3((unsigned)(total < cap ? total : cap)), dim3(256), S::NSTAGE * S::STAGE, s, g);
  return hipGetLastError();
}

// Which shape: measured with K = 256, 64-row tiles against 128-row tiles: 25.7 / 32.7 us for a 10752 x 256 update,
// 193 / 220 for 5376^2, 461 / 505 for the upper half of 10752^2, 3040 / 3038 for the upper half of 26624^2,
// 3245 / 3046 for 40960 x 8192.  The small tiles win while latencies matter and lose a little once the product is
// large enough to be bound by its traffic.
constexpr int64_t kI8SmallProduct = (int64_t)1 << 28;     // M * N up to here: 64-row tiles

hipError_t launch_gemm_i8s(const I8Operand& A, int a_row0, const I8Operand& B, int b_row0, double* C, int64_t ldc, int M,
                           int N, int K, double alpha, int beta, int upper_only, hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0) return hipSuccess;
  if (K > kI8MaxK || (a_row0 % 128) || (b_row0 % BN)) return hipErrorInvalidValue;
  return (int64_t)M * N <= kI8SmallProduct ? launch_shape<64>(A, a_row0, B, b_row0, C, ldc, M, N, K, alpha, beta, upper_only, s)
                                           : launch_shape<128>(A, a_row0, B, b_row0, C, ldc, M, N, K, alpha, beta, upper_only, s);
}

}  // namespace gptaq
