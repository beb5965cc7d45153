// Algorithm 1, lines 5-13 for one super-block of up to 1024 columns in a single launch.
//
// Rows of W never interact (Step 1: all output channels are solved in parallel with one shared
// factor), so a workgroup owns 64 rows for the whole super-block and needs no grid-level
// synchronisation: the 64 x 1024 slice of W lives in the accumulator registers of its four
// wavefronts from the first column of the super-block to the last, and every update of
// Eq. 15 / Eq. 18 that stays inside the super-block is applied there.
//
// Three levels of lazy batching (a re-association of the sums of Eq. 18, which leaves the result
// independent of the blocking):
//   * 16 columns ("sub-block"): the sequential column steps of lines 7-10, one row per lane, fp32
//     FMAs, the 16 x 16 diagonal pieces of U and P broadcast from LDS;
//   * the rest of the super-block: after each sub-block, W[:, later] += [-E | V] [U; P][sub-block, later]
//     on the matrix cores (bf16 hi/lo split of both sides, three products per term), straight into
//     the accumulators that hold W;
//   * the columns after the super-block: one GEMM per super-block, outside this kernel, from the
//     -E and V this kernel leaves behind in the GEMM's operand format.
//
// Who holds what.  The super-block is eight blocks of 128 columns; wave w holds blocks w and w + 4, each as
// four 32-column pieces of two 32 x 32 MFMA accumulator tiles (rows 0-31 and 32-63) of the TRANSPOSED
// product  W^T += [U; P]^T [-E | V]^T :  lane l, register v of a tile holds row l % 32 of the tile,
// column 8 (v / 4) + 4 (l / 32) + v % 4 of the piece.  v_permlane32_swap of the registers of the two
// tiles turns that into "one row per lane" for the sequential steps.
// While block b is worked on, the wave that holds it (the owner) runs the column steps of its eight
// sub-blocks and updates the rest of the block; the other three waves have no sequential work in
// that time: they apply each sub-block's update to the later blocks they hold, under the owner's next
// column steps.  One workgroup barrier per sub-block publishes its -E and V.
// The pieces are kept in a fixed place: the owner moves its pieces down by one when a piece is
// finished and its second block into the first one's registers when the block is finished, so every
// register index in the code is static.
#include "common.h"

namespace gptaq {

constexpr int kSbBlocks = kSbCols / 128;       // 128-column blocks per super-block
constexpr int kSub = 16;                       // columns per sub-block
constexpr int kSbEvents = kSbCols / kSub;      // sub-blocks per super-block

__device__ __forceinline__ uint16_t sb_bf16_rne(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ float sb_bf16_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Uniform affine min-max grid with 0 inside the range; the few operations per group are done in fp64 so
// that the fp32 scale is the correctly rounded (xmax - xmin) / maxq.
__device__ __forceinline__ void sb_grid_params(float xmin, float xmax, float maxq, int sym, float& scale, float& zero) {
  double lo = fmin((double)xmin, 0.0), hi = fmax((double)xmax, 0.0);
  if (sym) { hi = fmax(fabs(lo), hi); lo = -hi; }
  if (lo == 0.0 && hi == 0.0) { lo = -1.0; hi = 1.0; }
  scale = (float)((hi - lo) / (double)maxq);
  zero = sym ? (maxq + 1.f) * 0.5f : (float)rint(-lo / (double)scale);
}

// ---------------------------------------------------------------------------------------------------
// Left operands of the in-super-block updates: for sub-block e (rows sb0 + 16 e .. + 15 of U and P) and
// super-block column c, the 16 entries S[sb0 + 16 e + k][sb0 + c], k = 0..15, split into bf16 hi and lo, at
// out[(e * 1024 + c) * 16 + k]: the 32 columns x 16 k a wavefront needs for one MFMA operand are 1 KB in a row.
// grid (16, events, 2): blockIdx.x = tile of 64 columns, blockIdx.z = 0 for U, 1 for P.
__global__ __launch_bounds__(256) void near_operands_kernel(const float* U, const float* P, int64_t ldh, int n, int sb0,
                                                            uint16_t* Uh, uint16_t* Ul, uint16_t* Ph, uint16_t* Pl) {
  __shared__ float t[kSub][65];
  const int e = blockIdx.y, c0 = blockIdx.x * 64;
  if (c0 + 64 <= kSub * e) return;                         // entirely left of the sub-block: never read
  const float* S = blockIdx.z ? P : U;
  uint16_t* oh = blockIdx.z ? Ph : Uh;
  uint16_t* ol = blockIdx.z ? Pl : Ul;
  const int c = threadIdx.x & 63, kq = threadIdx.x >> 6;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int k = kq + 4 * p;
    const int64_t row = (int64_t)sb0 + kSub * e + k, col = (int64_t)sb0 + c0 + c;
    t[k][c] = (row < n && col < n) ? S[row * ldh + col] : 0.f;
  }
  __syncthreads();
  const int cc = threadIdx.x >> 2, k4 = (threadIdx.x & 3) * 4;
  uint16_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float v = t[k4 + i][cc];
    h[i] = sb_bf16_rne(v);
    l[i] = sb_bf16_rne(v - sb_bf16_f32(h[i]));
  }
  const int64_t o = ((int64_t)e * kSbCols + c0 + cc) * kSub + k4;
  u32x2 vh = {(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
  u32x2 vl = {(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
  *reinterpret_cast<u32x2*>(oh + o) = vh;
  *reinterpret_cast<u32x2*>(ol + o) = vl;
}

// ---------------------------------------------------------------------------------------------------
// Left operands of a sub-block's update, staged per wave: piece (32 columns) x {U hi, U lo, P hi, P lo} x 1 KB,
// written by global -> LDS loads one sub-block ahead of their use and read back by the lane that requested them.
constexpr int kSbPieces = 8;                     // per wave: 2 blocks x 4 pieces
constexpr int kSbStage = kSbPieces * 4 * 1024;
static_assert(kSbBlocks == 8, "two blocks per wave, four waves");
struct SbShared {
  // operands [-E | V]^T of a sub-block's update, in MFMA fragment order: [buffer][term][hi/lo][row half][k chunk][row]
  u32x4 frag[2][2][2][2][2][32];
  float Ud[2][kSub][kSub], Pd[2][kSub][kSub];     // diagonal pieces of U and P (fp32), double-buffered
  float dinv[2][kSub];                            // 1 / U_jj
};

// 1 KB per wavefront from global memory straight into LDS: lane l's 16 bytes land at lds + 16 l.
__device__ __forceinline__ void sb_load_lds(const uint16_t* src, unsigned char* lds) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                   (__attribute__((address_space(3))) void*)lds, 16, 0, 0);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding global
// store (the results a wave has just written, which nobody in this kernel reads back): a microsecond per
// sub-block.
__device__ __forceinline__ void sb_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Where this wave's pieces are while sub-block x is worked on.
struct SbGeo {
  int b, r, half, owner;      // block of the sub-block, finished pieces of that block, first/second half of a piece, owning wave
  int cur0;                   // block in slot 0 (the wave's first block until it has finished it, then its second)
  bool two;                   // slot 1 still holds the second block
  uint32_t active;            // bit 4 s + i: piece i of slot s takes the update of sub-block x
};
__device__ __forceinline__ SbGeo sb_geo(int x, int wave, int sbw, int nev, int terms) {
  SbGeo g;
  const int eb = x & 7;
  g.b = x >> 3; g.r = eb >> 1; g.half = eb & 1; g.owner = g.b & 3;
  g.cur0 = g.b > wave ? wave + 4 : wave;
  g.two = g.b <= wave;
  g.active = 0;
  if (terms != 0 && x + 1 < nev) {
    // pieces of block B that exist (the super-block may be narrower than 1024 columns)
    auto pieces_in = [&](int B) { return max(0, min(4, (sbw - 128 * B + 31) >> 5)); };
    uint32_t m0;
    if (g.cur0 == g.b) {
      // the block being worked on: its first g.r pieces are finished and have made room, so piece i is the block's
      // piece i + g.r; the piece the sub-block lies in takes the update of its second half only
      const int cnt = pieces_in(g.b) - g.r;
      m0 = cnt > 0 ? ((1u << cnt) - 1u) & ~(uint32_t)g.half : 0u;
    } else {
      m0 = g.cur0 > g.b ? (1u << pieces_in(g.cur0)) - 1u : 0u;
    }
    const uint32_t m1 = g.two ? (1u << pieces_in(wave + 4)) - 1u : 0u;     // (wave + 4 > b whenever slot 1 is in use)
    g.active = m0 | (m1 << 4);
  }
  return g;
}
// first super-block column of piece i of slot s
__device__ __forceinline__ int sb_piece_col(const SbGeo& g, int wave, int s, int i) {
  const int B = s == 0 ? g.cur0 : wave + 4;
  return 128 * B + 32 * (B == g.b ? i + g.r : i);
}

template <int HALF>
__device__ __forceinline__ void sb_extract(const f32x16 (&acc)[2][4][2], float (&w)[kSub]) {
  // registers 8 HALF .. 8 HALF + 7 of the current piece's two tiles -> the 16 columns of the sub-block, one row per lane
#pragma unroll
  for (int vv = 0; vv < 8; ++vv) {
    const float a0 = acc[0][0][0][8 * HALF + vv];
    const float a1 = acc[0][0][1][8 * HALF + vv];
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a0), __float_as_uint(a1), false, false);
    const int c = 8 * (vv >> 2) + (vv & 3);
    w[c] = __uint_as_float(r[0]);          // lanes 0-31: tile 0, lanes 32-63: tile 1, columns of lane half 0
    w[c + 4] = __uint_as_float(r[1]);      // the columns lane half 1 held
  }
}

// FAST: rows of W and of the codes are 16-byte aligned and n is a multiple of 16 (vector loads and stores).
template <bool FAST>
__global__ __launch_bounds__(256) void quant_sb_kernel(SbArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char sb_smem[];
  SbShared& sh = *reinterpret_cast<SbShared*>(sb_smem + 4 * kSbStage);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  unsigned char* const stage = sb_smem + wave * kSbStage;           // this wave's staged left operands
  const int l32 = lane & 31, lh = lane >> 5;
  const int row0 = blockIdx.x * 64;
  const int sbw = a.sbw;                                  // columns of this super-block
  const int nev = (sbw + kSub - 1) / kSub;
  const bool useE = a.terms & 1, useP = a.terms & 2;

  // ---- W -> accumulators.  Out-of-range elements read a clamped (valid) address and are replaced by 0,
  // so the loads need no branches.  Dead inputs were zeroed in W before this kernel.
  f32x16 acc[2][4][2];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int rh = 0; rh < 2; ++rh) {
        const int row = row0 + 32 * rh + l32;
        const float* src = a.W + (int64_t)min(row, a.m - 1) * a.ldw + a.sb0;
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int c = 128 * (wave + 4 * s) + 32 * i + 8 * vq + 4 * lh;    // super-block column of element 0
          if (FAST) {
            const bool ok = row < a.m && c < sbw;
            const f32x4 x = *reinterpret_cast<const f32x4*>(src + min(c, sbw - 4));
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[s][i][rh][4 * vq + q] = ok ? x[q] : 0.f;
          } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float x = src[min(c + q, sbw - 1)];
              acc[s][i][rh][4 * vq + q] = (row < a.m && c + q < sbw) ? x : 0.f;
            }
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);                  // (all 64 loads in flight at once would need 256 registers)
    }

  // ---- per-row grid (one row per lane); for grouped grids it is renewed by the owner at every group start
  float sc = 1.f, zr = 0.f, isc = 1.f;
  if (a.group <= 0) {
    const int row = row0 + lane;
    if (row < a.m) { sc = a.scales[row]; zr = a.zeros[row]; }
    isc = 1.f / sc;
  }

  // diagonal pieces of sub-block x into buffer x & 1: `which` 0 loads U (and 1 / U_jj), 1 loads P
  auto load_diag = [&](int x, int which) {
    const int j = lane >> 2, c4 = (lane & 3) * 4;
    const int64_t r = (int64_t)a.sb0 + kSub * x + j;
    const float* S = which ? a.P : a.U;
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t c = (int64_t)a.sb0 + kSub * x + c4 + i;
      const bool on = which ? useP : (useE || c4 + i == j);            // the diagonal of U is always needed
      v[i] = (on && r < a.n && c < a.n && c4 + i >= j && (which == 0 || c4 + i > j)) ? S[r * a.ldh + c] : 0.f;
    }
    float* dst = which ? &sh.Pd[x & 1][j][c4] : &sh.Ud[x & 1][j][c4];
    *reinterpret_cast<f32x4*>(dst) = f32x4{v[0], v[1], v[2], v[3]};
    if (which == 0 && (j >> 2) == (lane & 3)) {
      const float d = v[j & 3];
      sh.dinv[x & 1][j] = d != 0.f ? 1.f / d : 0.f;
    }
  };

  // Requests the left operands of sub-block x's update for this wave's pieces: they depend on U and P only, so
  // they are fetched a whole sub-block ahead (global -> LDS, no registers) and have the column steps' time to land.
  auto request_left = [&](int x, const SbGeo& g) {
    const uint32_t lane_off = (uint32_t)(l32 * kSub + 8 * lh);
    for (uint32_t rest = g.active; rest; rest &= rest - 1) {
      const int p = __builtin_ctz(rest);
      const int64_t o = ((int64_t)x * kSbCols + sb_piece_col(g, wave, p >> 2, p & 3)) * kSub + lane_off;
      unsigned char* dst = stage + p * 4096;
      if (useE) {
        sb_load_lds(a.Nop[0] + o, dst);
        sb_load_lds(a.Nop[1] + o, dst + 1024);
      }
      if (useP) {
        sb_load_lds(a.Nop[2] + o, dst + 2048);
        sb_load_lds(a.Nop[3] + o, dst + 3072);
      }
    }
  };
  SbGeo g_next = sb_geo(0, wave, sbw, nev, a.terms);
  request_left(0, g_next);
  if (wave == 1) load_diag(0, 0);
  if (wave == 2) load_diag(0, 1);
  __syncthreads();

  for (int e = 0; e < nev; ++e) {
    // (the lane number is re-read every iteration: addresses derived from it are then formed where they are
    // used instead of occupying registers through the whole loop, which has none to spare)
    int lane_v = lane;
    asm volatile("" : "+v"(lane_v));
    const SbGeo g = g_next;
    const int buf = e & 1;
    const int colg = a.sb0 + kSub * e;                    // first column of the sub-block
    const bool is_owner = wave == g.owner;

    // results of the 16 steps (owner only): W^ and the codes, packed one byte each as they are produced
    float wh[kSub];
    uint32_t cw[4] = {0u, 0u, 0u, 0u};
    if (is_owner) {
      const int row = row0 + lane_v;
      // ---- group range over the current (error-compensated) weights: the group's pieces are all in this wave
      if (a.group >= 32 && (kSub * e) % a.group == 0) {
        float mn[2], mx[2];
#pragma unroll
        for (int rh = 0; rh < 2; ++rh) {
          float lo = 0.f, hi = 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (32 * i < a.group) {
#pragma unroll
              for (int v = 0; v < 16; ++v) { lo = fminf(lo, acc[0][i][rh][v]); hi = fmaxf(hi, acc[0][i][rh][v]); }
            }
          const u32x2 r0 = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo), __float_as_uint(lo), false, false);
          const u32x2 r1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(hi), __float_as_uint(hi), false, false);
          mn[rh] = fminf(__uint_as_float(r0[0]), __uint_as_float(r0[1]));
          mx[rh] = fmaxf(__uint_as_float(r1[0]), __uint_as_float(r1[1]));
        }
        sb_grid_params(lh ? mn[1] : mn[0], lh ? mx[1] : mx[0], a.maxq, a.sym, sc, zr);
        isc = 1.f / sc;
        if (row < a.m) {
          const int64_t o = (int64_t)row * a.G + colg / a.group;
          a.scales[o] = sc;
          a.zeros[o] = zr;
        }
      }
      // ================= the 16 column steps of this sub-block (lines 7-10), one row per lane
      float w[kSub];
      if (g.half) sb_extract<1>(acc, w); else sb_extract<0>(acc, w);
      uint32_t peh[8], pel[8], pvh[8], pvl[8];             // -E and V as bf16 hi + lo pairs (operands of the updates)
      if (a.group == kSub) {                               // the group is this sub-block: its grid comes from the registers
        float mn = 0.f, mx = 0.f;
#pragma unroll
        for (int c = 0; c < kSub; ++c) { mn = fminf(mn, w[c]); mx = fmaxf(mx, w[c]); }
        sb_grid_params(mn, mx, a.maxq, a.sym, sc, zr);
        isc = 1.f / sc;
        if (row < a.m) {
          const int64_t o = (int64_t)row * a.G + colg / a.group;
          a.scales[o] = sc;
          a.zeros[o] = zr;
        }
      }
      const float* Ud = &sh.Ud[buf][0][0];
      const float* Pd = &sh.Pd[buf][0][0];
      // the pieces of row j of U and P right of the diagonal (and 1 / U_jj), fetched two steps ahead of their use: a
      // wait for "everything but the latest reads" then never waits for reads that have only just been issued
      f32x4 ub[3][4], pb[3][4];
      float db[3];
      auto fetch = [&](int j) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (4 * q + 3 > j) {
            ub[j % 3][q] = *reinterpret_cast<const f32x4*>(Ud + j * kSub + 4 * q);
            pb[j % 3][q] = *reinterpret_cast<const f32x4*>(Pd + j * kSub + 4 * q);
          }
        db[j % 3] = sh.dinv[buf][j];
      };
      fetch(0);
      fetch(1);
#pragma unroll
      for (int j = 0; j < kSub; ++j) {
        if (j + 2 < kSub) fetch(j + 2);
        const f32x4(&uc)[4] = ub[j % 3];
        const f32x4(&pc)[4] = pb[j % 3];
        const float dj = db[j % 3];
        const float v = w[j];
        // code - zero = clamp(rint(v / scale), -zero, maxq - zero): the same integers as clamp(rint(.) + zero, 0, maxq)
        // - zero, with a shorter dependency chain in front of the updates (one median instead of add, max, min, sub)
        const float d = __builtin_amdgcn_fmed3f(rintf(v * isc), -zr, a.maxq - zr);
        const float x = sc * d;
        const float e1 = (x - v) * dj;                    // -E_j
        wh[j] = x;
        cw[j >> 2] |= (uint32_t)(d + zr) << (8 * (j & 3));
        {
          const uint32_t h1 = sb_bf16_rne(e1), l1 = sb_bf16_rne(e1 - sb_bf16_f32((uint16_t)h1));
          const uint32_t h2 = sb_bf16_rne(v), l2 = sb_bf16_rne(v - sb_bf16_f32((uint16_t)h2));
          if (j & 1) { peh[j >> 1] |= h1 << 16; pel[j >> 1] |= l1 << 16; pvh[j >> 1] |= h2 << 16; pvl[j >> 1] |= l2 << 16; }
          else { peh[j >> 1] = h1; pel[j >> 1] = l1; pvh[j >> 1] = h2; pvl[j >> 1] = l2; }
        }
#pragma unroll
        for (int c = j + 1; c < kSub; ++c) w[c] = fmaf(e1, uc[c >> 2][c & 3], fmaf(v, pc[c >> 2][c & 3], w[c]));
      }
      {
        const int rh = lane >> 5;
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
          sh.frag[buf][0][0][rh][ch][l32] = u32x4{peh[4 * ch], peh[4 * ch + 1], peh[4 * ch + 2], peh[4 * ch + 3]};
          sh.frag[buf][0][1][rh][ch][l32] = u32x4{pel[4 * ch], pel[4 * ch + 1], pel[4 * ch + 2], pel[4 * ch + 3]};
          sh.frag[buf][1][0][rh][ch][l32] = u32x4{pvh[4 * ch], pvh[4 * ch + 1], pvh[4 * ch + 2], pvh[4 * ch + 3]};
          sh.frag[buf][1][1][rh][ch][l32] = u32x4{pvl[4 * ch], pvl[4 * ch + 1], pvl[4 * ch + 2], pvl[4 * ch + 3]};
        }
      }
      sb_barrier();
    } else {
      // the waves that hold later blocks fetch the next sub-block's diagonal pieces while they wait
      if (e + 1 < nev) {
        if (wave == ((g.owner + 1) & 3)) load_diag(e + 1, 0);
        if (wave == ((g.owner + 2) & 3)) load_diag(e + 1, 1);
      }
      sb_barrier();
    }

    // ================= every wave: this sub-block's update of its own later columns (Eq. 18 inside the super-block)
    if (g.active) {
      bf16x8 fe[2][2], fv[2][2];                          // [hi/lo][row half]
#pragma unroll
      for (int hl = 0; hl < 2; ++hl)
#pragma unroll
        for (int rh = 0; rh < 2; ++rh) {
          fe[hl][rh] = __builtin_bit_cast(bf16x8, sh.frag[buf][0][hl][rh][lh][l32]);
          fv[hl][rh] = __builtin_bit_cast(bf16x8, sh.frag[buf][1][hl][rh][lh][l32]);
        }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // the staged left operands (requested a sub-block ago) have landed
      const unsigned char* mine = stage + lane_v * 16;
      // one piece at a time, the next piece's operands read from LDS under this piece's MFMAs
      u32x4 cur[4];
      auto read_left = [&](int p, u32x4 (&dst)[4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (q < 2 ? useE : useP) dst[q] = *reinterpret_cast<const u32x4*>(mine + p * 4096 + q * 1024);
      };
      read_left(__builtin_ctz(g.active), cur);
#pragma unroll
      for (int p = 0; p < kSbPieces; ++p) {
        if ((g.active >> p) & 1u) {
          u32x4 nxt[4];
          const uint32_t rest = g.active >> (p + 1);
          if (rest) read_left(p + 1 + __builtin_ctz(rest), nxt);
          if (p == 0 && is_owner) {
            // the piece the sub-block lies in: the sub-block's own columns (its first half) take no update
            const bool keep = l32 >= kSub;
            const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int q = 0; q < 4; ++q) cur[q] = keep ? cur[q] : z;
          }
          f32x16(&t)[2] = acc[p >> 2][p & 3];
          if (useE) {
            const bf16x8 ah = __builtin_bit_cast(bf16x8, cur[0]), al = __builtin_bit_cast(bf16x8, cur[1]);
#pragma unroll
            for (int rh = 0; rh < 2; ++rh) {
              t[rh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, fe[0][rh], t[rh], 0, 0, 0);
              t[rh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, fe[1][rh], t[rh], 0, 0, 0);
              t[rh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, fe[0][rh], t[rh], 0, 0, 0);
            }
          }
          if (useP) {
            const bf16x8 ah = __builtin_bit_cast(bf16x8, cur[2]), al = __builtin_bit_cast(bf16x8, cur[3]);
#pragma unroll
            for (int rh = 0; rh < 2; ++rh) {
              t[rh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, fv[0][rh], t[rh], 0, 0, 0);
              t[rh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, fv[1][rh], t[rh], 0, 0, 0);
              t[rh] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, fv[0][rh], t[rh], 0, 0, 0);
            }
          }
#pragma unroll
          for (int q = 0; q < 4; ++q) cur[q] = nxt[q];
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    // the owner keeps its pieces in a fixed place: a finished piece makes room for the next, a finished block for
    // the wave's second block
    if (is_owner) {
      if ((e & 7) == 7) {
        if (g.two) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int rh = 0; rh < 2; ++rh) acc[0][i][rh] = acc[1][i][rh];
        }
      } else if (g.half) {
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
          for (int rh = 0; rh < 2; ++rh) acc[0][i][rh] = acc[0][i + 1][rh];
      }
    }
    // the staging area is free again (its reads have returned): request the next sub-block's operands, then let
    // this sub-block's results leave for memory
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    g_next = sb_geo(e + 1, wave, sbw, nev, a.terms);
    request_left(e + 1, g_next);
    if (is_owner) {
      const int row = row0 + lane_v;
      if (row < a.m) {
        float* wdst = a.W + (int64_t)row * a.ldw + colg;
        uint8_t* cdst = a.codes + (int64_t)row * a.n + colg;
        if (FAST) {
#pragma unroll
          for (int c4 = 0; c4 < kSub; c4 += 4)
            *reinterpret_cast<f32x4*>(wdst + c4) = f32x4{wh[c4], wh[c4 + 1], wh[c4 + 2], wh[c4 + 3]};
          *reinterpret_cast<u32x4*>(cdst) = u32x4{cw[0], cw[1], cw[2], cw[3]};
        } else {
#pragma unroll
          for (int c = 0; c < kSub; ++c)
            if (colg + c < a.n) { wdst[c] = wh[c]; cdst[c] = (uint8_t)(cw[c >> 2] >> (8 * (c & 3))); }
        }
      }
    }
    if (a.Eh && wave == ((g.owner + 3) & 3)) {
      // -E and V for the update of the columns after the super-block: copied to memory from the LDS fragments by
      // a wave that has nothing else to do now (they stay valid until the sub-block after next is published)
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int item = lane_v + 64 * it, r = item >> 1, ch = item & 1;
        if (row0 + r < a.m) {
          const int64_t o = (int64_t)(row0 + r) * a.ldev + kSub * e + 8 * ch;
          *reinterpret_cast<u32x4*>(a.Eh + o) = sh.frag[buf][0][0][r >> 5][ch][r & 31];
          *reinterpret_cast<u32x4*>(a.El + o) = sh.frag[buf][0][1][r >> 5][ch][r & 31];
          *reinterpret_cast<u32x4*>(a.Vh + o) = sh.frag[buf][1][0][r >> 5][ch][r & 31];
          *reinterpret_cast<u32x4*>(a.Vl + o) = sh.frag[buf][1][1][r >> 5][ch][r & 31];
        }
      }
    }
  }
}

hipError_t launch_near_operands(const float* U, const float* P, int64_t ldh, int n, int sb0, int sbw, uint16_t* const* N4,
                                hipStream_t s) {
  const int nev = (sbw + kSub - 1) / kSub;
  hipLaunchKernelGGL(near_operands_kernel, dim3(kSbCols / 64, nev, P ? 2 : 1), dim3(256), 0, s, U, P ? P : U, ldh, n, sb0,
                     N4[0], N4[1], N4[2], N4[3]);
  return hipGetLastError();
}

hipError_t launch_quant_sb(const SbArgs& a, hipStream_t s) {
  constexpr int lds = 4 * kSbStage + (int)sizeof(SbShared);
  static LdsLimitOnce fast_once, slow_once;
  hipError_t e = fast_once.ensure(reinterpret_cast<const void*>(&quant_sb_kernel<true>), lds);
  if (e == hipSuccess) e = slow_once.ensure(reinterpret_cast<const void*>(&quant_sb_kernel<false>), lds);
  if (e != hipSuccess) return e;
  if (a.fast_rows)
    hipLaunchKernelGGL(quant_sb_kernel<true>, dim3((a.m + 63) / 64), dim3(256), lds, s, a);
  else
    hipLaunchKernelGGL(quant_sb_kernel<false>, dim3((a.m + 63) / 64), dim3(256), lds, s, a);
  return hipGetLastError();
}

}  // namespace gptaq
