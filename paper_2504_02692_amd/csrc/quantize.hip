// Algorithm 1, lines 5-13: the blocked column loop and the lazy trailing update.
//
// Column loop (lines 7-10).  A wavefront owns R rows of W and keeps their slice of the
// active block (up to 128 columns) in registers, two columns per lane.  The block's
// U = L^T rows and P rows (128 x 128 fp32 each) live in LDS, shared by the workgroup's four
// wavefronts.  For column j the wave broadcasts v = W[r][j] out of the owning lane,
// quantises it (every lane redundantly, the value is wave-uniform), and each lane applies
//   W[r][j'] += -E_j U[j][j'] + v P[j][j']          (Eq. 15 in the form of Algorithm 1)
// to its two columns; U and P are zero left of the diagonal so no lane masking is needed.
// Group ranges are wave reductions (min/max over the lanes that hold the group).
// The kernel leaves the quantised block in W, the codes, and -E and V (the pre-quantisation
// columns) split into bf16 hi+lo as the left operand of the trailing GEMM.
//
// Trailing update (lines 11-12, Eq. 18):  W[:, i+B:] += [-E | V] [U; P][i:i+B, i+B:] on the
// MFMA GEMM with three bf16 cross products per term (operands carried to about 2^-17 relative, fp32 sums).
#include "common.h"
#include <mutex>

namespace gptaq {

constexpr int QB = 128;                       // widest block the column-loop kernel holds
constexpr int Q_LDS = 2 * QB * QB * 4 + QB * 4;

__device__ __forceinline__ uint16_t q_bf16_rne(float f) {
  __bf16 b = (__bf16)f;
  return __builtin_bit_cast(uint16_t, b);
}
__device__ __forceinline__ float q_bf16_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Uniform affine min-max grid with 0 inside the range.  The few operations per group are done
// in fp64 so that the fp32 scale is the correctly rounded (xmax - xmin) / maxq.
__device__ __forceinline__ void grid_params(float xmin, float xmax, float maxq, int sym, float& scale, float& zero) {
  double lo = fmin((double)xmin, 0.0), hi = fmax((double)xmax, 0.0);
  if (sym) { hi = fmax(fabs(lo), hi); lo = -hi; }
  if (lo == 0.0 && hi == 0.0) { lo = -1.0; hi = 1.0; }
  scale = (float)((hi - lo) / (double)maxq);
  zero = sym ? (maxq + 1.f) * 0.5f : (float)rint(-lo / (double)scale);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Clip-range search (Section 5.1: the clipping range of the weights is the one with the smallest squared
// quantisation error): candidates shrink the min-max range by p = 1 - i / grid, i = 0 .. steps - 1, about its
// zero-point, i.e. scale_i = fp32(p * scale_0 exact) with the zero-point of the full range; the
// candidate with the smallest sum of squared errors over the group wins, the earlier one on ties.
struct ClipSearch {
  double base;      // (hi - lo) / maxq, not yet rounded
  float zero, maxq;
  float best_err, best_scale;
  __device__ __forceinline__ void begin(float xmin, float xmax, float mq, int sym) {
    double lo = fmin((double)xmin, 0.0), hi = fmax((double)xmax, 0.0);
    if (sym) { hi = fmax(fabs(lo), hi); lo = -hi; }
    if (lo == 0.0 && hi == 0.0) { lo = -1.0; hi = 1.0; }
    base = (hi - lo) / (double)mq;
    maxq = mq;
    zero = sym ? (mq + 1.f) * 0.5f : (float)rint(-lo / (double)(float)base);
    best_err = __builtin_inff();
    best_scale = (float)base;
  }
  __device__ __forceinline__ float scale_of(int i, int grid) const { return (float)((1.0 - (double)i / (double)grid) * base); }
  __device__ __forceinline__ float err_of(float x, float sc, float isc) const {
    const float q = fminf(fmaxf(rintf(x * isc) + zero, 0.f), maxq);
    const float d = sc * (q - zero) - x;
    return d * d;
  }
  __device__ __forceinline__ void offer(float err, float sc) {
    if (err < best_err) { best_err = err; best_scale = sc; }
  }
};

// One wavefront per row: range of the whole (original) row -> one (scale, zero) per row.
__global__ __launch_bounds__(256) void row_params_kernel(const float* W, int64_t ldw, int m, int n, const uint8_t* dead,
                                                         float maxq, int sym, int mse_grid, int mse_steps, float* scales,
                                                         float* zeros) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= m) return;
  float mn = 0.f, mx = 0.f;
  for (int c = lane; c < n; c += 64) {
    float v = W[(int64_t)row * ldw + c];
    if (dead && dead[c]) v = 0.f;
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
  mn = wave_min(mn);
  mx = wave_max(mx);
  float sc, zr;
  grid_params(mn, mx, maxq, sym, sc, zr);
  if (mse_steps > 0) {
    ClipSearch cs;
    cs.begin(mn, mx, maxq, sym);
    for (int i = 0; i < mse_steps; ++i) {
      const float si = cs.scale_of(i, mse_grid), isi = 1.f / si;
      float e = 0.f;
      for (int c = lane; c < n; c += 64) {
        float v = W[(int64_t)row * ldw + c];
        if (dead && dead[c]) v = 0.f;
        e += cs.err_of(v, si, isi);
      }
      cs.offer(wave_sum(e), si);
    }
    sc = cs.best_scale;
    zr = cs.zero;
  }
  if (lane == 0) { scales[row] = sc; zeros[row] = zr; }
}

struct QuantArgs {
  float* W; int64_t ldw; int m, n, i0, bw;
  const float* U; const float* P; int64_t ldh;
  const uint8_t* dead;
  float maxq; int group, sym, G, terms;        // terms: bit 0 = E term, bit 1 = P term of Eq. 15
  int mse_grid, mse_steps;                     // clip-range search (0 steps: plain min-max)
  float* scales; float* zeros; uint8_t* codes;
  uint16_t *Eh, *El, *Vh, *Vl;          // bf16 hi/lo of -E and V: row stride ldev, this block's 128 slots at evoff
  int64_t ldev; int evoff;
};

template <int R, int NW>
__global__ __launch_bounds__(64 * NW) void quant_block_kernel(QuantArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  float* Us = reinterpret_cast<float*>(smem_raw);
  float* Ps = Us + QB * QB;
  float* dinv = Ps + QB * QB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i0 = a.i0, bw = a.bw;

  for (int idx = tid; idx < QB * QB; idx += 64 * NW) {
    const int r = idx >> 7, c = idx & 127;
    float u = 0.f, p = 0.f;
    if (r < bw && c < bw && c >= r) {
      const int64_t o = (int64_t)(i0 + r) * a.ldh + i0 + c;
      if (c == r || (a.terms & 1)) u = a.U[o];          // the diagonal is always needed (E divides by it)
      if (c > r && (a.terms & 2)) p = a.P[o];
    }
    Us[idx] = u;
    Ps[idx] = p;
  }
  if (tid < QB) dinv[tid] = tid < bw ? 1.f / a.U[(int64_t)(i0 + tid) * a.ldh + i0 + tid] : 0.f;

  const int row0 = (blockIdx.x * NW + wave) * R;
  // w: the row's current values of the lane's two columns; v: the value each column had just before it
  // was quantised; (sc, zr): the current group's grid (wave-uniform); (ms, mz): the grid of the group
  // the lane's own columns belong to.  Codes and -E are recomputed per lane after the loop from
  // (v, ms, mz), with the same fp32 operations the loop used, so nothing else has to be captured.
  float w0[R], w1[R], v0[R], v1[R], sc[R], zr[R], isc[R], ms0[R], mz0[R], ms1[R], mz1[R];
  const bool col0 = lane < bw && !(a.dead && a.dead[i0 + lane]);
  const bool col1 = lane + 64 < bw && !(a.dead && a.dead[i0 + 64 + lane]);
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = row0 + r;
    const bool ok = row < a.m;
    w0[r] = ok && col0 ? a.W[(int64_t)row * a.ldw + i0 + lane] : 0.f;
    w1[r] = ok && col1 ? a.W[(int64_t)row * a.ldw + i0 + 64 + lane] : 0.f;
    v0[r] = v1[r] = 0.f;
    sc[r] = 1.f; zr[r] = 0.f;
    if (a.group <= 0 && ok) { sc[r] = a.scales[row]; zr[r] = a.zeros[row]; }
    isc[r] = 1.f / sc[r];
    ms0[r] = ms1[r] = sc[r];
    mz0[r] = mz1[r] = zr[r];
  }
  __syncthreads();

  int next_group = a.group > 0 ? 0 : bw;                  // i0 is a multiple of the group size
  auto group_start = [&](int j) {
    const int jend = j + a.group;
    const bool in0 = lane >= j && lane < jend, in1 = lane + 64 >= j && lane + 64 < jend;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float mn = fminf(in0 ? w0[r] : 0.f, in1 ? w1[r] : 0.f);
      float mx = fmaxf(in0 ? w0[r] : 0.f, in1 ? w1[r] : 0.f);
      mn = wave_min(mn);
      mx = wave_max(mx);
      grid_params(mn, mx, a.maxq, a.sym, sc[r], zr[r]);
      if (a.mse_steps > 0) {
        ClipSearch cs;
        cs.begin(mn, mx, a.maxq, a.sym);
        for (int i = 0; i < a.mse_steps; ++i) {
          const float si = cs.scale_of(i, a.mse_grid), isi = 1.f / si;
          const float e = (in0 ? cs.err_of(w0[r], si, isi) : 0.f) + (in1 ? cs.err_of(w1[r], si, isi) : 0.f);
          cs.offer(wave_sum(e), si);
        }
        sc[r] = cs.best_scale;
        zr[r] = cs.zero;
      }
      isc[r] = 1.f / sc[r];
      if (in0) { ms0[r] = sc[r]; mz0[r] = zr[r]; }
      if (in1) { ms1[r] = sc[r]; mz1[r] = zr[r]; }
      const int row = row0 + r;
      if (lane == 0 && row < a.m) {
        const int64_t o = (int64_t)row * a.G + (i0 + j) / a.group;
        a.scales[o] = sc[r];
        a.zeros[o] = zr[r];
      }
    }
    next_group += a.group;
  };

  const int h1 = bw < 64 ? bw : 64;
  for (int j = 0; j < h1; ++j) {                           // columns held in w0
    if (j == next_group) group_start(j);
    const float u0 = Us[j * QB + lane], u1 = Us[j * QB + 64 + lane];
    const float p0 = Ps[j * QB + lane], p1 = Ps[j * QB + 64 + lane];
    const float dj = dinv[j];
    const bool mine = lane == j;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w0[r]), j));
      const float q = fminf(fmaxf(rintf(v * isc[r]) + zr[r], 0.f), a.maxq);
      const float wh = sc[r] * (q - zr[r]);
      const float ne = (wh - v) * dj;                     // -E_j
      const float n0 = fmaf(v, p0, fmaf(ne, u0, w0[r]));
      w1[r] = fmaf(v, p1, fmaf(ne, u1, w1[r]));
      w0[r] = mine ? wh : n0;
      v0[r] = mine ? v : v0[r];
    }
  }
  for (int j = 64; j < bw; ++j) {                          // columns held in w1; w0 is final
    if (j == next_group) group_start(j);
    const float u1 = Us[j * QB + 64 + lane], p1 = Ps[j * QB + 64 + lane];
    const float dj = dinv[j];
    const bool mine = lane == j - 64;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(w1[r]), j - 64));
      const float q = fminf(fmaxf(rintf(v * isc[r]) + zr[r], 0.f), a.maxq);
      const float wh = sc[r] * (q - zr[r]);
      const float ne = (wh - v) * dj;
      const float n1 = fmaf(v, p1, fmaf(ne, u1, w1[r]));
      w1[r] = mine ? wh : n1;
      v1[r] = mine ? v : v1[r];
    }
  }

  const float d0 = dinv[lane], d1 = dinv[64 + lane];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = row0 + r;
    if (row >= a.m) continue;
    const float q0 = fminf(fmaxf(rintf(v0[r] * (1.f / ms0[r])) + mz0[r], 0.f), a.maxq);
    const float q1 = fminf(fmaxf(rintf(v1[r] * (1.f / ms1[r])) + mz1[r], 0.f), a.maxq);
    const float e0 = (w0[r] - v0[r]) * d0, e1 = (w1[r] - v1[r]) * d1;       // -E; 0 in the padding
    if (lane < bw) {
      a.W[(int64_t)row * a.ldw + i0 + lane] = w0[r];
      a.codes[(int64_t)row * a.n + i0 + lane] = (uint8_t)q0;
    }
    if (lane + 64 < bw) {
      a.W[(int64_t)row * a.ldw + i0 + 64 + lane] = w1[r];
      a.codes[(int64_t)row * a.n + i0 + 64 + lane] = (uint8_t)q1;
    }
    const int64_t o = (int64_t)row * a.ldev + a.evoff + lane;
    uint16_t h;
    h = q_bf16_rne(e0); a.Eh[o] = h; a.El[o] = q_bf16_rne(e0 - q_bf16_f32(h));
    h = q_bf16_rne(e1); a.Eh[o + 64] = h; a.El[o + 64] = q_bf16_rne(e1 - q_bf16_f32(h));
    h = q_bf16_rne(v0[r]); a.Vh[o] = h; a.Vl[o] = q_bf16_rne(v0[r] - q_bf16_f32(h));
    h = q_bf16_rne(v1[r]); a.Vh[o + 64] = h; a.Vl[o + 64] = q_bf16_rne(v1[r] - q_bf16_f32(h));
  }
}

// Right operands of a trailing GEMM: for each of the `gridDim.z` column blocks (chunk c covers the rows
// sb0 + c * blocksize .. of U and P), the entries in the columns [c_begin, c_end), transposed to
// (column x K) with the chunk's rows at K offsets 128 c .. 128 c + 127 (zero padded), split into bf16 hi+lo.
// grid (ceil(padded columns / 64), 2, chunks): blockIdx.y = 0 for U, 1 for P.
__device__ __forceinline__ void split_transpose_rows_tile(const float* S, int64_t ldh, int n, int sb0, int blocksize,
                                                          int chunk, int c_begin, int c_end, uint16_t* oh, uint16_t* ol,
                                                          int64_t ldo) {
  __shared__ uint16_t th[64][QB + 2], tl[64][QB + 2];
  const int i0 = sb0 + chunk * blocksize;
  const int bw = min(blocksize, n - i0);
  const int j0 = blockIdx.x * 64;
  const int c = threadIdx.x & 63, kq = threadIdx.x >> 6;
  const int col = c_begin + j0 + c;
  for (int p = 0; p < QB / 4; ++p) {
    const int kk = kq + 4 * p;
    float v = 0.f;
    if (kk < bw && col < c_end) v = S[(int64_t)(i0 + kk) * ldh + col];
    const uint16_t h = q_bf16_rne(v);
    th[c][kk] = h;
    tl[c][kk] = q_bf16_rne(v - q_bf16_f32(h));
  }
  __syncthreads();
  // 64 rows x 128 bf16 = 64 x 64 dwords; thread t writes dword (t & 63) of rows (t >> 6) + 4p
  const int d = threadIdx.x & 63;
  for (int p = 0; p < 16; ++p) {
    const int r = (threadIdx.x >> 6) + 4 * p;
    const uint32_t vh = (uint32_t)th[r][2 * d] | ((uint32_t)th[r][2 * d + 1] << 16);
    const uint32_t vl = (uint32_t)tl[r][2 * d] | ((uint32_t)tl[r][2 * d + 1] << 16);
    reinterpret_cast<uint32_t*>(oh + (int64_t)(j0 + r) * ldo + chunk * QB)[d] = vh;
    reinterpret_cast<uint32_t*>(ol + (int64_t)(j0 + r) * ldo + chunk * QB)[d] = vl;
  }
}

__global__ __launch_bounds__(256) void split_transpose_rows_kernel(const float* U, const float* P, int64_t ldh, int n,
                                                                   int sb0, int blocksize, int c_begin, int c_end,
                                                                   uint16_t* Uth, uint16_t* Utl, uint16_t* Pth,
                                                                   uint16_t* Ptl, int64_t ldo) {
  split_transpose_rows_tile(blockIdx.y ? P : U, ldh, n, sb0, blocksize, blockIdx.z, c_begin, c_end,
                            blockIdx.y ? Pth : Uth, blockIdx.y ? Ptl : Utl, ldo);
}

// Rows of the far right operands of super-block k: its columns after the super-block, in whole 256-row GEMM tiles,
// plus one tile of zero rows (a 256-tile whose first row is the last 128-tile's reads that far).
__host__ __device__ inline int64_t far_rows(int64_t n, int k) {
  const int64_t rest = n - (int64_t)(k + 1) * kSbCols;
  return (rest + 255) / 256 * 256 + 256;
}

// The far right operands of EVERY super-block that has columns after it, in one launch: they depend on U and P only,
// so nothing of this has to sit between two super-blocks.  Super-block k's operands start at row sum_{i<k} far_rows(i)
// of the four output arrays (row stride kSbCols); row r of its part holds column (k + 1) * kSbCols + r.
// grid (far_rows(0) / 64, 2, 8 * number of such super-blocks): blockIdx.z = 8 k + chunk of 128 rows of the super-block.
__global__ __launch_bounds__(256) void far_operands_all_kernel(const float* U, const float* P, int64_t ldh, int n,
                                                               uint16_t* Uth, uint16_t* Utl, uint16_t* Pth,
                                                               uint16_t* Ptl) {
  const int k = blockIdx.z / (kSbCols / QB), chunk = blockIdx.z % (kSbCols / QB);
  if ((int64_t)blockIdx.x * 64 >= far_rows(n, k)) return;
  int64_t first = 0;
  for (int i = 0; i < k; ++i) first += far_rows(n, i);
  const int64_t o = first * kSbCols;
  split_transpose_rows_tile(blockIdx.y ? P : U, ldh, n, k * kSbCols, QB, chunk, (k + 1) * kSbCols, n,
                            (blockIdx.y ? Pth : Uth) + o, (blockIdx.y ? Ptl : Utl) + o, (int64_t)kSbCols);
}

}  // namespace gptaq

using namespace gptaq;

namespace {
constexpr int SB = 8;                         // column blocks per super-block (two-level lazy batching; 2, 4, 16 measured slower)
constexpr int KS = SB * QB;
struct QLayout {
  int64_t mp, np;
  size_t off[24], off_far[4], total;
};
QLayout q_layout(int64_t m, int64_t n) {
  QLayout L;
  L.mp = round_up(m, 256);
  L.np = round_up(n, 256);
  size_t o = 0;
  for (int i = 0; i < 24; ++i) {
    L.off[i] = o;
    // 0-3: -E, V (hi, lo) of one super-block; 4-7: right operands of the updates of one super-block as the
    // block-per-wave path makes them (all columns from the super-block's first on, plus a tile of padding rows);
    // 8-11: left operands of the updates inside a super-block (quantize_sb.hip); 12-15 and 20-23: a second set of 0-3
    // and 8-11 (the far update of a super-block runs beside the next super-block, which writes its own -E and V; or
    // the two row halves of a tall matrix run as two chains, each at its own super-block); 16-19: unused
    const int k = i < 12 ? i : i - 12;
    o += (size_t)(k < 4 ? L.mp * KS * 2 : k < 8 ? (i < 12 ? (L.np + 256) * KS * 2 : 0) : (int64_t)(kSbCols / 16) * kSbCols * 16 * 2);
  }
  // the far right operands of every super-block of the layer (far_operands_all_kernel), made once per call
  int64_t rows = 0;
  for (int k = 0; (int64_t)(k + 1) * kSbCols < n; ++k) rows += far_rows(n, k);
  for (int i = 0; i < 4; ++i) { L.off_far[i] = o; o += (size_t)rows * kSbCols * 2; }
  L.total = o;
  return L;
}

// rows from which a matrix is quantised as two row halves (measured: 8192 x 4096 1.89 -> 1.95 ms, 8192 x 8192
// 5.68 -> 5.49, 10240 x 8192 6.68 -> 6.08, 12288 x 4096 2.44 -> 2.21, 22016 x 4096 4.44 -> 3.57)
constexpr int64_t kRowSplitMin = 10240;

template <int R, int NW>
hipError_t launch_quant(const QuantArgs& a, hipStream_t s) {
  static LdsLimitOnce lds_once;                  // per instantiation
  {
    const hipError_t e = lds_once.ensure((const void*)&quant_block_kernel<R, NW>, Q_LDS);
    if (e != hipSuccess) return e;
  }
  const int rows_per_wg = NW * R;
  hipLaunchKernelGGL((quant_block_kernel<R, NW>), dim3((a.m + rows_per_wg - 1) / rows_per_wg), dim3(64 * NW), Q_LDS, s, a);
  return hipGetLastError();
}
// Rows are spread over the 256 CUs with two wavefronts per SIMD where m allows it (the loop is a
// dependency chain; the second wavefront hides its latencies).
hipError_t launch_quant_for(const QuantArgs& a, hipStream_t s) {
  const int m = a.m;
  if (m <= 1024) return launch_quant<1, 4>(a, s);
  const int r = (m + 2047) / 2048;
  if (r <= 1) return launch_quant<1, 8>(a, s);
  if (r <= 2) return launch_quant<2, 8>(a, s);
  if (r <= 3) return launch_quant<3, 8>(a, s);
  if (r <= 4) return launch_quant<4, 8>(a, s);
  if (r <= 6) return launch_quant<6, 8>(a, s);
  if (r <= 8) return launch_quant<8, 8>(a, s);
  // up to 24576 rows still fit one round of workgroups (a second round would run less than half full)
  if (r <= 10) return launch_quant<10, 8>(a, s);
  if (r <= 12) return launch_quant<12, 8>(a, s);
  return launch_quant<8, 8>(a, s);
}
}  // namespace

extern "C" size_t gptaq_quantize_workspace_bytes(int64_t m, int64_t n) {
  if (m <= 0 || n <= 0) return 0;
  return q_layout(m, n).total;
}

namespace gptaq {
// Dead inputs (zero Hessian diagonal): their columns of W count as 0 (GPTQ's rule, which the paper defers to).
// grid: one workgroup per 64 columns; it returns at once unless one of its columns is dead.
__global__ __launch_bounds__(256) void zero_dead_columns_kernel(float* W, int64_t ldw, int m, int n, const uint8_t* dead) {
  __shared__ int any;
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const bool d = c < n && dead[c];
  if (threadIdx.x == 0) any = 0;
  __syncthreads();
  if (d) any = 1;
  __syncthreads();
  if (!any) return;
  for (int r = threadIdx.x >> 6; r < m; r += 4)
    if (d) W[(int64_t)r * ldw + c] = 0.f;
}
}  // namespace gptaq

// Algorithm 1, lines 5-13 with one launch of quant_sb_kernel per super-block (column steps and every update
// inside the super-block) followed by the update of the columns after it (Eq. 18) on the MFMA GEMM.  The result does
// not depend on the blocking (Eq. 18 only re-associates sums), so the caller's blocksize is not used here.
//
// Two chains.  Super-block k + 1 only needs the far update of super-block k on ITS OWN columns; the update of the
// columns after it has until super-block k + 2 starts.  So the far update is split by columns: "far1" (the next
// super-block's columns) stays on the caller's stream, "far2" (everything after) runs on the library's helper stream
// beside super-block k + 1, which mostly leaves the chip idle (its length is set by the chain of column steps, and a
// 4096-row layer fills 64 of the 256 CUs).  Every column still receives its updates in super-block order (far1(k)
// waits for far2(k - 1), which touches the same columns), so results are bit-reproducible.  -E and V are
// double-buffered: far2(k) reads set k & 1 while super-block k + 1 writes the other.  The right operands of all far
// updates (`farop`) are made once per call, before the first super-block: they depend on U and P only, and a split
// pass between two super-blocks sat on the critical path of every one of them (4096 x 11008: 5.8 -> 4.9 ms).
static int quantize_layer_sb(float* W, int64_t m, int64_t n, int64_t ldw, const float* U, const float* P, int64_t ldh,
                             const uint8_t* dead, int bits, int group, int sym, uint8_t* codes, float* scales,
                             float* zeros, uint16_t* const* buf, uint16_t* const* farop, hipStream_t s, int terms,
                             bool may_use_helper = true, bool make_farop = true) {
  constexpr int64_t LDE = kSbCols;               // row stride of the -E / V buffers and of the far right operands
  if (dead) {
    hipLaunchKernelGGL(zero_dead_columns_kernel, dim3((unsigned)((n + 63) / 64)), dim3(256), 0, s, W, ldw, (int)m, (int)n, dead);
    GPTAQ_LAUNCH_CHECK();
  }
  SbArgs a;
  a.W = W; a.ldw = ldw; a.m = (int)m; a.n = (int)n;
  a.U = U; a.P = (terms & 2) ? P : U; a.ldh = ldh;
  for (int i = 0; i < 4; ++i) a.Nop[i] = buf[8 + i];
  a.dead = dead;
  a.maxq = (float)((1 << bits) - 1); a.group = group; a.sym = sym; a.terms = terms;
  a.G = group > 0 ? (int)(n / group) : 1;
  a.scales = scales; a.zeros = zeros; a.codes = codes;
  a.ldev = LDE;
  a.fast_rows = (ldw % 4 == 0) && (((uintptr_t)W & 15) == 0) && (n % 16 == 0) && (((uintptr_t)codes & 15) == 0);
  if (group <= 0) {
    hipLaunchKernelGGL(row_params_kernel, dim3((unsigned)((m + 3) / 4)), dim3(256), 0, s, W, ldw, (int)m, (int)n,
                       (const uint8_t*)nullptr, a.maxq, sym, 0, 0, scales, zeros);
    GPTAQ_LAUNCH_CHECK();
  }
  const int nsb = (int)((n + kSbCols - 1) / kSbCols);
  // (with one or two super-blocks there is no far2; it pays when the super-block kernel leaves most of the chip free:
  // measured on 4096 x 11008, 6.50 -> 5.77 ms, but 12288 x 4096 with a quarter of the chip for far2, 2.41 -> 2.90 ms)
  int cus = 256, dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 256;
  const int sbk_wgs = (int)((m + 63) / 64);
  const bool two_chains = may_use_helper && terms != 0 && nsb >= 3 && sbk_wgs <= cus / 4;
  std::unique_lock<std::mutex> side_lock(side_stream_mutex(), std::defer_lock);
  SideStream* side = nullptr;
  if (two_chains) {
    side_lock.lock();
    side = side_stream(3 * nsb + 3);
    if (!side) { set_last_hip_error(hipGetLastError()); return GPTAQ_ELAUNCH; }
  }
  bool ok = true;
  auto chk = [&](hipError_t e) { if (e != hipSuccess && ok) { ok = false; set_last_hip_error(e); } };
  if (make_farop && terms != 0 && nsb >= 2) {
    // right operands of every far update: rows of U and P of each super-block, the columns after it, transposed to
    // (column x K) and split into bf16 hi + lo; a GEMM reads whole tiles of rows, hence the zero rows past n.  With two
    // chains the pass runs on the helper stream, beside the first super-block.
    hipStream_t st = s;
    if (two_chains) {
      st = side->stream;
      chk(hipEventRecord(side->events[2 * nsb + 1], s));             // (U and P are ready where the caller's stream stands)
      chk(hipStreamWaitEvent(st, side->events[2 * nsb + 1], 0));
    }
    {
      ProfScope ps(kProfTrailSplit, st);
      hipLaunchKernelGGL(far_operands_all_kernel, dim3((unsigned)(far_rows(n, 0) / 64), 2, (unsigned)((nsb - 1) * (kSbCols / QB))),
                         dim3(256), 0, st, U, (terms & 2) ? P : U, ldh, (int)n, farop[0], farop[1], farop[2], farop[3]);
      chk(hipGetLastError());
    }
    if (two_chains) chk(hipEventRecord(side->events[2 * nsb + 2], st));
  }
  auto ev_sbk = [&](int k) { return side->events[2 * k]; };       // super-block k's kernel has finished
  auto ev_far2 = [&](int k) { return side->events[2 * k + 1]; };  // its far2 update has finished
  // W[:, c0:c1] += [-E | V] [U; P][super-block rows, c0:c1]: -E and V from buffer set `set`, the right operands of
  // super-block k from `farop` (made for the whole layer before the first super-block; row 0 of k's part is column cbase)
  auto far_update = [&](int set, int k, int64_t c0, int64_t c1, int64_t cbase, hipStream_t st, int max_wgs) {
    uint16_t* const* ev = buf + (set ? 12 : 0);
    int64_t first = 0;
    for (int i = 0; i < k; ++i) first += far_rows(n, i);
    const uint16_t* rop[4];
    for (int i = 0; i < 4; ++i) rop[i] = farop[i] + first * LDE;
    const int64_t nt = c1 - c0, ro = (c0 - cbase) * LDE;
    const int tile = gemm_tile_for(m, nt);
    GemmBatch b{};
    b.nprob = 1; b.tile = tile; b.max_wgs = max_wgs;
    GemmProblem& g = b.p[0];
    g.C = W + c0; g.ldc = ldw; g.M = (int)m; g.N = (int)nt; g.K = kSbCols;
    g.tiles_m = (int)(round_up(m, tile) / tile); g.tiles_n = (int)(round_up(nt, tile) / tile);
    g.kind = 2; g.nterm = 0; g.tile_mode = 0; g.k_mode = 0; g.store_mode = 0;
    if (terms & 1) g.term[g.nterm++] = {{ev[0], ev[1]}, {rop[0] + ro, rop[1] + ro}, LDE, LDE, 32, 32};
    if (terms & 2) g.term[g.nterm++] = {{ev[2], ev[3]}, {rop[2] + ro, rop[3] + ro}, LDE, LDE, 32, 32};
    ProfScope ps(kProfTrailGemm, st);
    chk(launch_gemm(b, st));
  };
  for (int k = 0; k < nsb && ok; ++k) {
    const int64_t sb0 = (int64_t)k * kSbCols;
    const int64_t sb_end = n < sb0 + kSbCols ? n : sb0 + kSbCols;
    const bool far = terms != 0 && sb_end < n;
    const int set = two_chains ? (k & 1) : 0;
    uint16_t* const* ev = buf + (set ? 12 : 0);
    a.sb0 = (int)sb0; a.sbw = (int)(sb_end - sb0);
    a.Eh = far ? ev[0] : nullptr; a.El = ev[1]; a.Vh = ev[2]; a.Vl = ev[3];
    // this super-block's columns must have every earlier update, and its buffer set must be free again
    if (two_chains && k >= 2) chk(hipStreamWaitEvent(s, ev_far2(k - 2), 0));
    if (terms != 0) {
      ProfScope ps(kProfTrailSplit, s);
      chk(launch_near_operands(U, (terms & 2) ? P : nullptr, ldh, (int)n, (int)sb0, a.sbw, buf + 8, s));
    }
    {
      ProfScope ps(kProfColumnLoop, s);
      chk(launch_quant_sb(a, s));
    }
    if (!far) continue;
    const int64_t next_end = n < sb_end + kSbCols ? n : sb_end + kSbCols;
    const bool has_far2 = two_chains && next_end < n;
    // While far2 is long (many columns left) it sets the pace and starts at once, sharing the chip with far1; once it
    // is shorter than a super-block it only slows far1 down, which the next super-block waits for: then it starts
    // when far1 is done.
    // (measured on 4096 x 11008 with the switch at 0 / 2 / 4 / 6 / 10 super-blocks of columns left: 5.66 / 5.62 / 5.60 /
    // 5.54 / 5.68 ms; 4096 x 4096: 1.59 / 1.53 / 1.50 / 1.51 / 1.50)
    constexpr int kFar2LateCols = 6 * kSbCols;
    const bool far2_late = has_far2 && (n - next_end) <= kFar2LateCols;
    auto launch_far2 = [&]() {
      chk(hipEventRecord(ev_sbk(k), s));
      chk(hipStreamWaitEvent(side->stream, ev_sbk(k), 0));
      // far2: beside the next super-block, on the compute units that one leaves free (a 256-tile fills a unit, two
      // 128-tiles share one)
      far_update(set, k, next_end, n, sb_end, side->stream, (cus - sbk_wgs) * (gemm_tile_for(m, n - next_end) == 256 ? 1 : 2));
      chk(hipEventRecord(ev_far2(k), side->stream));
    };
    if (has_far2 && !far2_late) launch_far2();
    if (two_chains && k >= 1) chk(hipStreamWaitEvent(s, ev_far2(k - 1), 0));   // it adds to the same columns: keep the order
    if (two_chains && k == 0 && make_farop) chk(hipStreamWaitEvent(s, side->events[2 * nsb + 2], 0));   // the far operands
    far_update(set, k, sb_end, two_chains ? next_end : n, sb_end, s, 0);   // far1: the next super-block's columns (or all of them)
    if (far2_late) launch_far2();
  }
  if (two_chains) {
    // whatever was handed to the helper stream is behind the caller's stream when the call returns, error or not
    const hipError_t keep = (hipError_t)gptaq_last_hip_error();
    hipEvent_t ev_join = side->events[2 * nsb];
    if (hipEventRecord(ev_join, side->stream) == hipSuccess) hipStreamWaitEvent(s, ev_join, 0);
    if (!ok) set_last_hip_error(keep);
  }
  return ok ? GPTAQ_OK : GPTAQ_ELAUNCH;
}

static int quantize_layer_impl(float* W, int64_t m, int64_t n, int64_t ldw, const float* U, const float* P,
                               int64_t ldh, const uint8_t* dead, int bits, int group, int sym, int blocksize,
                               uint8_t* codes, float* scales, float* zeros, void* ws, size_t ws_bytes,
                               void* stream, int terms, int mse_grid, int mse_steps) {
  if (!W || !U || (!P && (terms & 2)) || !codes || !scales || !zeros || !ws) return GPTAQ_ENULL;
  if (terms < 0 || terms > 3 || mse_steps < 0 || (mse_steps > 0 && (mse_grid <= 0 || mse_steps > mse_grid)))
    return GPTAQ_EUNSUPPORTED;
  if (m <= 0 || n <= 0 || ldw < n || ldh < n || m > (1 << 24) || n > (1 << 24)) return GPTAQ_EDIM;
  if (bits < 2 || bits > 8 || blocksize < 1 || blocksize > QB) return GPTAQ_EUNSUPPORTED;
  if (group > 0 && (n % group || blocksize % group || group > QB)) return GPTAQ_EUNSUPPORTED;
  if ((uintptr_t)ws & 255) return GPTAQ_EWORKSPACE;
  const QLayout L = q_layout(m, n);
  if (ws_bytes < L.total) return GPTAQ_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  unsigned char* base = (unsigned char*)ws;
  uint16_t* buf[24];
  for (int i = 0; i < 24; ++i) buf[i] = (uint16_t*)(base + L.off[i]);

  // The super-block kernel takes groups that tile its 16/32/128-column pieces; the clip-range search and other
  // group sizes go through the block-by-block kernels below.
  if (mse_steps == 0 && (group <= 0 || group == 16 || group == 32 || group == 64 || group == 128)) {
    // Rows are independent (Step 1).  A tall matrix goes through as two row halves on two streams: the super-block
    // kernel of one half, whose length is a chain of column steps whatever the number of rows, then runs beside the
    // far update of the other half instead of leaving the chip to it alone (and 344 workgroups of 64 rows no
    // longer make a second, mostly empty round on 256 CUs).
    const int64_t nsb = (n + kSbCols - 1) / kSbCols;
    uint16_t* farop[4];
    for (int i = 0; i < 4; ++i) farop[i] = (uint16_t*)(base + L.off_far[i]);
    if (terms != 0 && nsb >= 2 && m >= kRowSplitMin) {
      {
        // the far operands serve both halves: made once, before the streams fork
        ProfScope ps(kProfTrailSplit, s);
        hipLaunchKernelGGL(far_operands_all_kernel, dim3((unsigned)(far_rows(n, 0) / 64), 2, (unsigned)((nsb - 1) * (kSbCols / QB))),
                           dim3(256), 0, s, U, (terms & 2) ? P : U, ldh, (int)n, farop[0], farop[1], farop[2], farop[3]);
        GPTAQ_LAUNCH_CHECK();
      }
      const int64_t mA = round_up((m + 1) / 2, 256), mB = m - mA;   // (a multiple of the GEMM's row tile: the halves' padded
                                                                    //  rows of the -E / V buffers then do not overlap)
      const int64_t G = group > 0 ? n / group : 1;
      std::lock_guard<std::mutex> side_lock(side_stream_mutex());
      SideStream* side = side_stream(2);
      if (!side) { set_last_hip_error(hipGetLastError()); return GPTAQ_ELAUNCH; }
      hipEvent_t ev_fork = side->events[0], ev_join = side->events[1];
      if (hipEventRecord(ev_fork, s) != hipSuccess || hipStreamWaitEvent(side->stream, ev_fork, 0) != hipSuccess) {
        set_last_hip_error(hipGetLastError());
        return GPTAQ_ELAUNCH;
      }
      uint16_t* bufB[12];
      for (int i = 0; i < 4; ++i) bufB[i] = buf[i] + mA * kSbCols;          // its rows of the -E / V buffers
      for (int i = 4; i < 12; ++i) bufB[i] = buf[12 + i];                  // operands of its own
      const int rcB = quantize_layer_sb(W + mA * ldw, mB, n, ldw, U, P, ldh, dead, bits, group, sym, codes + mA * n,
                                        scales + mA * G, zeros + mA * G, bufB, farop, side->stream, terms, false, false);
      const int rcA = quantize_layer_sb(W, mA, n, ldw, U, P, ldh, dead, bits, group, sym, codes, scales, zeros, buf, farop,
                                        s, terms, false, false);
      // the helper stream is behind the caller's stream when the call returns, error or not
      const hipError_t keep = (hipError_t)gptaq_last_hip_error();
      if (hipEventRecord(ev_join, side->stream) == hipSuccess) hipStreamWaitEvent(s, ev_join, 0);
      if (rcA != GPTAQ_OK || rcB != GPTAQ_OK) set_last_hip_error(keep);
      return rcA != GPTAQ_OK ? rcA : rcB;
    }
    return quantize_layer_sb(W, m, n, ldw, U, P, ldh, dead, bits, group, sym, codes, scales, zeros, buf, farop, s, terms);
  }

  QuantArgs a;
  a.W = W; a.ldw = ldw; a.m = (int)m; a.n = (int)n;
  a.U = U; a.P = P; a.ldh = ldh; a.dead = dead;
  a.maxq = (float)((1 << bits) - 1); a.group = group; a.sym = sym; a.terms = terms; a.mse_grid = mse_grid; a.mse_steps = mse_steps;
  a.G = group > 0 ? (int)(n / group) : 1;
  a.scales = scales; a.zeros = zeros; a.codes = codes;
  a.Eh = buf[0]; a.El = buf[1]; a.Vh = buf[2]; a.Vl = buf[3]; a.ldev = KS;

  if (group <= 0) {
    hipLaunchKernelGGL(row_params_kernel, dim3((unsigned)((m + 3) / 4)), dim3(256), 0, s, W, ldw, (int)m, (int)n, dead,
                       a.maxq, sym, mse_grid, mse_steps, scales, zeros);
    GPTAQ_LAUNCH_CHECK();
  }
  // Two-level lazy batching (a re-association of the sums of Eq. 18): a block's update reaches the rest
  // of its super-block at once ("near", K = one block), and the columns after the super-block once per
  // super-block ("far", K = SB blocks), which cuts the passes over W of the flat schedule by SB.
  // The right operands (rows of U and P of the super-block, transposed and split into bf16 hi + lo) are
  // made once per super-block for every column from its first on: row c - sb0 of R4[.] holds column c, the
  // rows of block p at K offsets 128 p ...  Near and far updates read their part of it.
  uint16_t* const* R4 = buf + 4;
  auto trailing = [&](int64_t c0, int64_t c1, const uint16_t* const* L4, int64_t sb0, int koff, int K) -> int {
    if (terms == 0) return GPTAQ_OK;                    // no update at all: round to nearest
    const int64_t nt = c1 - c0;
    const int tile = gemm_tile_for(m, nt);
    const int64_t ntp = round_up(nt, tile);
    const int64_t ro = (c0 - sb0) * KS + koff;
    GemmBatch b{};
    b.nprob = 1; b.tile = tile;
    GemmProblem& g = b.p[0];
    g.C = W + c0; g.ldc = ldw; g.M = (int)m; g.N = (int)nt; g.K = K;
    g.tiles_m = (int)(round_up(m, tile) / tile); g.tiles_n = (int)(ntp / tile);
    g.kind = 2; g.nterm = 0; g.tile_mode = 0; g.k_mode = 0; g.store_mode = 0;
    if (terms & 1) g.term[g.nterm++] = {{L4[0], L4[1]}, {R4[0] + ro, R4[1] + ro}, KS, KS, 32, 32};
    if (terms & 2) g.term[g.nterm++] = {{L4[2], L4[3]}, {R4[2] + ro, R4[3] + ro}, KS, KS, 32, 32};
    hipError_t e;
    {
      ProfScope ps(kProfTrailGemm, s);
      e = launch_gemm(b, s);
    }
    if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
    return GPTAQ_OK;
  };
  for (int64_t sb0 = 0; sb0 < n; sb0 += (int64_t)SB * blocksize) {
    const int64_t sb_end = n < sb0 + (int64_t)SB * blocksize ? n : sb0 + (int64_t)SB * blocksize;
    const int nb = (int)((sb_end - sb0 + blocksize - 1) / blocksize);
    if (terms != 0 && sb0 + blocksize < n) {
      ProfScope ps(kProfTrailSplit, s);
      const int64_t rows = round_up(n - sb0, 256) + 256;   // a trailing GEMM reads whole tiles of rows: zeros past n
      hipLaunchKernelGGL(split_transpose_rows_kernel, dim3((unsigned)(rows / 64), 2, (unsigned)nb), dim3(256), 0, s,
                         U, (terms & 2) ? P : U, ldh, (int)n, (int)sb0, blocksize, (int)sb0, (int)n, R4[0], R4[1], R4[2],
                         R4[3], (int64_t)KS);
      GPTAQ_LAUNCH_CHECK();
    }
    for (int p = 0; p < nb; ++p) {
      const int64_t i0 = sb0 + (int64_t)p * blocksize;
      const int bw = (int)(n - i0 < blocksize ? n - i0 : blocksize);
      const int64_t i2 = i0 + bw;
      a.i0 = (int)i0; a.bw = bw; a.evoff = p * QB;
      {
        ProfScope ps(kProfColumnLoop, s);
        hipError_t e = launch_quant_for(a, s);
        if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
      }
      if (i2 < sb_end) {
        const uint16_t* L4[4] = {a.Eh + p * QB, a.El + p * QB, a.Vh + p * QB, a.Vl + p * QB};
        const int rc = trailing(i2, sb_end, L4, sb0, p * QB, QB);
        if (rc != GPTAQ_OK) return rc;
      }
    }
    if (sb_end < n) {
      const uint16_t* L4[4] = {a.Eh, a.El, a.Vh, a.Vl};
      const int rc = trailing(sb_end, n, L4, sb0, 0, nb * QB);
      if (rc != GPTAQ_OK) return rc;
    }
  }
  return GPTAQ_OK;
}

extern "C" int gptaq_quantize_layer(float* W, int64_t m, int64_t n, int64_t ldw, const float* U, const float* P,
                                    int64_t ldh, const uint8_t* dead, int bits, int group, int sym, int blocksize,
                                    uint8_t* codes, float* scales, float* zeros, void* ws, size_t ws_bytes,
                                    void* stream) {
  return quantize_layer_impl(W, m, n, ldw, U, P, ldh, dead, bits, group, sym, blocksize, codes, scales, zeros, ws,
                             ws_bytes, stream, 3, 0, 0);
}

extern "C" int gptaq_quantize_layer_terms(float* W, int64_t m, int64_t n, int64_t ldw, const float* U, const float* P,
                                          int64_t ldh, const uint8_t* dead, int bits, int group, int sym,
                                          int blocksize, uint8_t* codes, float* scales, float* zeros, void* ws,
                                          size_t ws_bytes, void* stream, int terms) {
  return quantize_layer_impl(W, m, n, ldw, U, P, ldh, dead, bits, group, sym, blocksize, codes, scales, zeros, ws,
                             ws_bytes, stream, terms, 0, 0);
}

extern "C" int gptaq_quantize_layer_ex(float* W, int64_t m, int64_t n, int64_t ldw, const float* U, const float* P,
                                       int64_t ldh, const uint8_t* dead, int bits, int group, int sym, int blocksize,
                                       uint8_t* codes, float* scales, float* zeros, void* ws, size_t ws_bytes,
                                       void* stream, int terms, int mse_grid, int mse_steps) {
  return quantize_layer_impl(W, m, n, ldw, U, P, ldh, dead, bits, group, sym, blocksize, codes, scales, zeros, ws,
                             ws_bytes, stream, terms, mse_grid, mse_steps);
}
