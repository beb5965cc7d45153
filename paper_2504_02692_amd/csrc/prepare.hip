// Algorithm 1, lines 3-4: damping, the inverse-Cholesky factor and the fused matrix P.
//
// Step 3 of the paper needs L with (H + lambda I)^-1 = L L^T.  Instead of inverting and then
// factoring, factor  H + lambda I = V V^T  with V UPPER triangular (a Cholesky factorisation
// run from the last row/column towards the first); then U = L^T = V^-1 (the factor is unique
// for a positive diagonal).  Factorisation and triangular inverse are swept together from the
// bottom-right to the top-left, in fp64, inside one n x n fp64 array F whose strictly-upper
// region holds Schur-complement data until its block column is factored and the running
// right-hand side R of the solve V U = I afterwards.  Two block levels:
//
//   for every outer block OB of 256 columns, last to first      (I: rows above OB, J: columns right of OB)
//     ob     : ONE launch, one workgroup (ob_factor_kernel), for the 256 x 256 diagonal block of OB; for every inner
//              block K of 64 columns in OB, last to first:
//       diag   : F_KK = V_KK V_KK^T   (one wavefront; Winv_K = V_KK^-1 by another, beside the solves)
//       panel  : V_iK = F_iK V_KK^-T  for the row tiles i of OB above K (triangular solves, one row per lane)
//       inner  : F_ij -= V_iK V_jK^T  for the tiles (i <= j) of OB left of K (rank 64), the next diagonal tile first
//     tall   : the same panels (as products with Winv_K) and rank-64 updates for the rows above OB, one launch
//     syrk   : F_II  -= V_I,OB V_I,OB^T                (rank 256)  } the n^3 * 2/3 bulk: digit-sliced operands,
//     trinv  : U_OB,OB = V_OB,OB^-1  from the Winv_K and the V_kj inside OB          exact int8 MFMA products,
//     rowblk : U_OB,J  = U_OB,OB R_OB,J                                              fp64 recombination
//     rupd   : R_I,J  -= V_I,OB U_OB,J                 (rank 256)  }                 (gemm_i8s.hip)
//     close  : R_I,OB  = -V_I,OB U_OB,OB
//
// Theorem 4.2's two products then run on the bf16 MFMA GEMM with fp32 operands split into
// bf16 hi+lo (three cross products per term).
#include "common.h"
#include <mutex>
#include <vector>

namespace gptaq {

constexpr int NB = 64;
typedef __attribute__((ext_vector_type(2))) double f64x2;
constexpr int LDT = 66;                       // padded LDS row (doubles); even, so that two entries are one 16-byte read
constexpr int MM_LDS = 2 * NB * LDT * 8;      // bytes for two staged tiles

constexpr int NBO = 256;                      // outer block (columns per rank-256 update)

struct Sweep {
  double* F;
  int64_t ldf;
  int n, kb, nblk;
  double* Dinv;      // nblk tiles of 64 x 64: V_KK^-1
  int32_t* info;
  int o0, o1, jlo;   // current outer block [o0, o1); first inner block of it
  double* Uob;       // 256 x 256 scratch: U_OB,OB
  double* Vob;       // 256 x 256 scratch: the V_iK with i inside OB (tile row i - jlo, tile column K - jlo)
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
// A NaN or Inf in the upper triangle of H is reported as info[0] = -(1 + row of the entry) (smallest row wins).
__global__ void build_F_kernel(const float* H, int64_t ldh, int n, const double* lam, double* F, int64_t ldf, int32_t* info) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x, i = blockIdx.y;
  if (j >= n || j < i) return;
  const float h = H[(int64_t)i * ldh + j];
  if (!__builtin_isfinite(h)) atomicMin(info, -(1 + i));
  double v = (double)h;
  if (i == j) { if (v == 0.0) v = 1.0; v += *lam; }
  F[(int64_t)i * ldf + j] = v;
}

// ------------------------------------------------------------------- 64 x 64 x 64 in LDS
// out[i][c] = sum_l A[i][l] * B[l][c] with As[l*LDT + i], Bs[l*LDT + c]; thread (ty, tx)
// owns rows 4ty..4ty+3 and columns 2tx, 2tx+1, 32+2tx, 33+2tx (mm_col), so that its four entries of a row of
// As and of Bs are two 16-byte LDS reads each and the 16 threads tx of a row read 16 consecutive 16-byte pieces
// (no bank conflicts; four consecutive columns per thread would put tx and tx+8 on the same banks).
// The operand reads run ahead of the products in register sets of their own: left to itself the compiler reads
// into the same registers every step and waits for them before the first product (~150 clocks per step, 10K per
// product); one step ahead 131, three steps ahead 123 clocks per step = 7.9K clocks per product, which is what the
// four wavefronts' operand reads (16 KB per step at 128 B per clock) allow; the 16 v_fma_f64 of a step issue in ~75.
__device__ __forceinline__ constexpr int mm_col(int tx, int q) { return (q >> 1) * 32 + 2 * tx + (q & 1); }
struct MmRegs { f64x2 a0, a1, b0, b1; };
__device__ __forceinline__ void mm64_read(MmRegs& r, const double* pa, const double* pb) {
  r.a0 = *reinterpret_cast<const f64x2*>(pa);
  r.a1 = *reinterpret_cast<const f64x2*>(pa + 2);
  r.b0 = *reinterpret_cast<const f64x2*>(pb);
  r.b1 = *reinterpret_cast<const f64x2*>(pb + 32);
}
template <bool SUB>
__device__ __forceinline__ void mm64_mul(const MmRegs& r, double (&acc)[4][4]) {
  const double a[4] = {SUB ? -r.a0[0] : r.a0[0], SUB ? -r.a0[1] : r.a0[1], SUB ? -r.a1[0] : r.a1[0], SUB ? -r.a1[1] : r.a1[1]};
  const double b[4] = {r.b0[0], r.b0[1], r.b1[0], r.b1[1]};
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[p][q] = fma(a[p], b[q], acc[p][q]);
}
// DEEP: reads three steps ahead (four register sets) instead of one: 16 products (~75 clocks) are shorter than an
// LDS round trip.  Reads past the last step fetch the last step again, so that they need no branch (a conditional
// read costs a second copy of the register set and moves).
template <bool SUB, bool DEEP>
__device__ __forceinline__ void mm64_core(const double* As, const double* Bs, double (&acc)[4][4]) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const double* pa = As + 4 * ty;
  const double* pb = Bs + 2 * tx;
  auto at = [](int l) { return (l < NB ? l : NB - 1) * LDT; };
  if (!DEEP) {
    MmRegs r0, r1;
    mm64_read(r0, pa, pb);
#pragma clang loop unroll(disable)
    for (int l = 0; l < NB; l += 2) {
      mm64_read(r1, pa + (l + 1) * LDT, pb + (l + 1) * LDT);
      __builtin_amdgcn_sched_barrier(0);
      mm64_mul<SUB>(r0, acc);
      __builtin_amdgcn_sched_barrier(0);
      mm64_read(r0, pa + at(l + 2), pb + at(l + 2));
      __builtin_amdgcn_sched_barrier(0);
      mm64_mul<SUB>(r1, acc);
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    MmRegs r0, r1, r2, r3;
    mm64_read(r0, pa, pb);
    mm64_read(r1, pa + LDT, pb + LDT);
    mm64_read(r2, pa + 2 * LDT, pb + 2 * LDT);
#pragma clang loop unroll(disable)
    for (int l = 0; l < NB; l += 4) {
      mm64_read(r3, pa + (l + 3) * LDT, pb + (l + 3) * LDT);
      __builtin_amdgcn_sched_barrier(0);
      mm64_mul<SUB>(r0, acc);
      __builtin_amdgcn_sched_barrier(0);
      mm64_read(r0, pa + at(l + 4), pb + at(l + 4));
      __builtin_amdgcn_sched_barrier(0);
      mm64_mul<SUB>(r1, acc);
      __builtin_amdgcn_sched_barrier(0);
      mm64_read(r1, pa + at(l + 5), pb + at(l + 5));
      __builtin_amdgcn_sched_barrier(0);
      mm64_mul<SUB>(r2, acc);
      __builtin_amdgcn_sched_barrier(0);
      mm64_read(r2, pa + at(l + 6), pb + at(l + 6));
      __builtin_amdgcn_sched_barrier(0);
      mm64_mul<SUB>(r3, acc);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

__device__ __forceinline__ void mm64(const double* As, const double* Bs, double (&acc)[4][4]) {
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[p][q] = 0.0;
  mm64_core<false, true>(As, Bs, acc);
}

// acc[i][c] -= sum_l A[i][l] * B[l][c], same layouts (the running tile is the accumulator: no second register tile)
constexpr bool MM_SUB_DEEP = true;
__device__ __forceinline__ void mm64_sub(const double* As, const double* Bs, double (&acc)[4][4]) {
  mm64_core<true, MM_SUB_DEEP>(As, Bs, acc);
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

// fast fp64 reciprocal: hardware estimate + two Newton steps (about 1 ulp; no correctly rounded divide needed here)
__device__ __forceinline__ double fast_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = fma(fma(-x, r, 1.0), r, r);
  r = fma(fma(-x, r, 1.0), r, r);
  return r;
}
// ------------------------------------------------------------------------------- diag
// One wavefront: reverse Cholesky of the 64 x 64 diagonal block and the inverse of its factor, with no
// workgroup barrier inside the sequential steps.  Lane r keeps row r of the symmetric block S in registers
// (both triangles).  At step j a lane downdates its column c with S[r][j] S[c][j] / S[j][j], so it needs the
// whole pivot column; by symmetry lane c holds S[c][j] in its own register j, so ONE LDS store (every lane
// its own entry) publishes the column and all lanes read it back at the same addresses (broadcast reads).
// Column j is final when step j starts and is never touched again; columns are scaled at the end.
// The inverse W of the factor V is built the same way from W V = I, column by column: column c of V is
// published with one store, W[r][c] = -(sum_{l < c} W[r][l] V[l][c]) / V[c][c] needs only the lane's own
// row of W (entries left of the diagonal are zero, so the sum may start at 0).
// LDS written by some lanes of the wavefront becomes readable by the others: to the compiler the store
// and the loads are ordered by a wavefront-scope fence (without it the exchange is a data race, and the
// loads do get moved ahead of the store); to the hardware they already are (one wavefront, in order).
__device__ __forceinline__ void wave_publish() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The two halves are separate functions for one wavefront each, because only the factor is on the critical
// path of the sweep: the panels inside the outer block are triangular solves with V (solve_wave), and the inverse
// is made by another wavefront meanwhile.
// cholesky_wave: LDS T (NB * LDV doubles; rows of LDT doubles while the block is staged, of LDV afterwards),
// colb (2 * NB), dsh (NB).  Leaves Vt[c * LDV + l] = V[l][c] for l <= c in T and dsh[c] = 1 / V[c][c].
constexpr int LDV = NB + 2;                   // even row stride: a column of V is read two entries at a time
constexpr int DIAG_LDS_DOUBLES = NB * LDV + 2 * NB + NB;
// On entry T holds the block row-major (row stride LDT; only the upper triangle is read), padded with the
// identity where the matrix ends; k0 = index of the block's first column (for the report of a bad pivot).
// Reads of a column of V (LDS, wave-uniform addresses) in inverse_wave and solve_wave go through a ring of RD batches
// of 8 entries: a batch is requested RD-1 batches before it is used, which covers the LDS latency with the
// products of the batches in between (one batch ahead did not: 16 products are shorter than a round trip).
// All indices are compile-time constants once the loops are unrolled.
constexpr int RQ = 4;                          // f64x2 per batch
constexpr int RD = 6;                          // ring depth (solve, inverse)

__device__ __forceinline__ double lane_value(double v, int l) {       // v of lane l (l a constant), wave-uniform
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)b, l), hi = __builtin_amdgcn_readlane((uint32_t)(b >> 32), l);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ void cholesky_wave(const Sweep& a, double* T, double* colb0, double* dsh, int k0) {
  double* colb[2] = {colb0, colb0 + NB};
  const int lane = threadIdx.x & 63;
  double s[NB];
#pragma unroll
  for (int c = 0; c < NB; ++c) s[c] = c >= lane ? T[lane * LDT + c] : T[c * LDT + lane];   // mirrored into rows
  wave_publish();                                                 // (T is rewritten with another row stride below)
  double piv = 1.0;                                               // S[lane][lane] when its step starts
  // Step j downdates with pivot column j: s[c] += nci * cb[c] for c < j, nci = -S[lane][j] / S[j][j], cb[c] =
  // S[c][j] = lane c's entry of column j.  The chain from one step to the next is: downdate column j-1, take its
  // pivot and the entries of lanes j-2 and j-3 out of the registers (v_readlane: no LDS round trip), reciprocal,
  // next nci.  The other columns [0, j-2) need the whole pivot column in every lane: it is published through LDS
  // when it is final (one step earlier), read at the top of the step and used around the reciprocal.
  constexpr int QH = NB / 4;                                      // f64x2 per half column
  colb[(NB - 1) & 1][lane] = s[NB - 1];
  double nci, c1, c2;
  {
    const double sjj = lane_value(s[NB - 1], NB - 1);
    c1 = lane_value(s[NB - 1], NB - 2);
    c2 = lane_value(s[NB - 1], NB - 3);
    const bool bad = !(sjj > 0.0);
    if (bad && lane == 0) atomicCAS(a.info, 0, k0 + NB);
    piv = lane == NB - 1 ? sjj : piv;
    nci = -(s[NB - 1] * (bad ? 0.0 : fast_rcp(sjj)));
  }
  wave_publish();
#pragma clang loop unroll(full)
  for (int j = NB - 1; j >= 1; --j) {
    const double* cb = colb[j & 1];
    double* nb = colb[(j - 1) & 1];
    const int rest = j - 2;                                       // columns [0, rest) beside the two done first
    f64x2 q[QH];
#pragma unroll
    for (int u = 0; u < QH; ++u)
      if (2 * u < rest) q[u] = *reinterpret_cast<const f64x2*>(cb + 2 * u);
    __builtin_amdgcn_sched_barrier(0);
    s[j - 1] = fma(nci, c1, s[j - 1]);
    nb[lane] = s[j - 1];
    if (j >= 2) s[j - 2] = fma(nci, c2, s[j - 2]);
    const double sjj = lane_value(s[j - 1], j - 1);
    if (j >= 2) c1 = lane_value(s[j - 1], j - 2);
    if (j >= 3) c2 = lane_value(s[j - 1], j - 3);
    const bool bad = !(sjj > 0.0);
    if (bad && lane == 0) atomicCAS(a.info, 0, k0 + j);
    piv = lane == j - 1 ? sjj : piv;
    const double nci_next = -(s[j - 1] * (bad ? 0.0 : fast_rcp(sjj)));
#pragma unroll
    for (int u = 0; u < QH; ++u) {
      if (2 * u < rest) s[2 * u] = fma(nci, q[u][0], s[2 * u]);
      if (2 * u + 1 < rest) s[2 * u + 1] = fma(nci, q[u][1], s[2 * u + 1]);
    }
    if (rest > 2 * QH) {                                          // second half of a long column
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < QH; ++u)
        if (2 * QH + 2 * u < rest) q[u] = *reinterpret_cast<const f64x2*>(cb + 2 * QH + 2 * u);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < QH; ++u) {
        const int m = 2 * QH + 2 * u;
        if (m < rest) s[m] = fma(nci, q[u][0], s[m]);
        if (m + 1 < rest) s[m + 1] = fma(nci, q[u][1], s[m + 1]);
      }
    }
    nci = nci_next;
    wave_publish();                                               // column j-1 is readable from here on
  }
  // V[i][j] = S[i][j] / sqrt(S[j][j]) for i <= j; 1 / V[j][j] is the same factor.  All columns of V are
  // published at once: Vt[c][l] = V[l][c] (entries below the diagonal are garbage and are not read).
  double* Vt = T;
  dsh[lane] = piv > 0.0 ? 1.0 / sqrt(piv) : 1.0;
  wave_publish();
#pragma unroll
  for (int c = 0; c < NB; ++c) Vt[c * LDV + lane] = s[c] * dsh[c];
  wave_publish();
}

// inverse_wave: W = V^-1 from Vt and dsh as cholesky_wave leaves them; lane r gets row r of W in wv:
// W[r][c] = -(sum_{l < c} W[r][l] V[l][c]) / V[c][c] column by column (entries left of the diagonal are zero, so
// the sum may start at 0).
__device__ __forceinline__ void inverse_wave(const double* Vt, const double* dsh, double (&wv)[NB]) {
  const int lane = threadIdx.x & 63;
  f64x2 q[RD][RQ];
  int pc = 1, ph = 0, pslot = 0;                           // next batch to request: column pc, entries [8 ph, 8 ph + 8)
  auto request = [&]() {
    if (pc < NB) {
#pragma unroll
      for (int u = 0; u < RQ; ++u)
        if (2 * RQ * ph + 2 * u < pc) q[pslot][u] = *reinterpret_cast<const f64x2*>(Vt + pc * LDV + 2 * RQ * ph + 2 * u);
      pslot = (pslot + 1) % RD;
      if (2 * RQ * (ph + 1) < pc) ++ph; else { ++pc; ph = 0; }
    }
  };
#pragma unroll
  for (int d = 0; d < RD - 1; ++d) request();
  int cur = 0;
  double dc = dsh[0];
#pragma clang loop unroll(full)
  for (int c = 0; c < NB; ++c) {
    double p0 = 0.0, p1 = 0.0, p2 = 0.0, p3 = 0.0;
    const double dcur = dc;
    if (c + 1 < NB) dc = dsh[c + 1];
#pragma unroll
    for (int h = 0; h < NB / (2 * RQ); ++h) {
      if (2 * RQ * h >= c) continue;
      request();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < RQ; u += 2) {
        const int l = 2 * RQ * h + 2 * u;
        if (l < c) p0 = fma(wv[l], q[cur][u][0], p0);
        if (l + 1 < c) p1 = fma(wv[l + 1], q[cur][u][1], p1);
        if (l + 2 < c) p2 = fma(wv[l + 2], q[cur][u + 1][0], p2);
        if (l + 3 < c) p3 = fma(wv[l + 3], q[cur][u + 1][1], p3);
      }
      // (the sums are only used by the lanes right of the diagonal; left alone, the compiler moves all the products
      //  of a column into that branch, behind the reads of all its batches)
      asm volatile("" : "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3));
      __builtin_amdgcn_sched_barrier(0);
      cur = (cur + 1) % RD;
    }
    wv[c] = lane == c ? dcur : (lane < c ? -dcur * ((p0 + p1) + (p2 + p3)) : 0.0);
  }
}

// solve_wave: X V^T = Fin for a 64 x 64 tile, V upper triangular as cholesky_wave leaves it (Vt, dsh).  Lane r
// holds row r: X[r][l] = (Fin[r][l] - sum_{m > l} X[r][m] V[l][m]) / V[l][l], columns from the last to the
// first; as soon as X[r][l] is known it is taken out of the columns left of l (V[c][l], c < l, is column l of V).
// Fin is row-major in LDS (row stride LDT) and is only read by this wavefront; the result goes back into the same
// buffer in the left/right-operand layout of mm64: Xk[l * LDT + r] = X[r][l].
__device__ __forceinline__ void solve_wave(const double* Vt, const double* dsh, double* buf) {
  const int lane = threadIdx.x & 63;
  double f[NB];
#pragma unroll
  for (int c = 0; c < NB; ++c) f[c] = buf[lane * LDT + c];
  wave_publish();                                         // every lane has its row before the buffer is overwritten
  f64x2 q[RD][RQ];
  int pl = NB - 1, ph = 0, pslot = 0;                      // next batch to request: column pl, entries [8 ph, 8 ph + 8)
  auto request = [&]() {
    if (pl >= 1) {
#pragma unroll
      for (int u = 0; u < RQ; ++u)
        if (2 * RQ * ph + 2 * u < pl) q[pslot][u] = *reinterpret_cast<const f64x2*>(Vt + pl * LDV + 2 * RQ * ph + 2 * u);
      pslot = (pslot + 1) % RD;
      if (2 * RQ * (ph + 1) < pl) ++ph; else { --pl; ph = 0; }
    }
  };
#pragma unroll
  for (int d = 0; d < RD - 1; ++d) request();
  int cur = 0;
  double dl = dsh[NB - 1];
#pragma clang loop unroll(full)
  for (int l = NB - 1; l >= 0; --l) {
    const double x = f[l] * dl;
    buf[l * LDT + lane] = x;
    if (l > 0) dl = dsh[l - 1];
#pragma unroll
    for (int h = 0; h < NB / (2 * RQ); ++h) {
      if (2 * RQ * h >= l) continue;
      request();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < RQ; ++u) {
        const int m = 2 * RQ * h + 2 * u;
        if (m < l) f[m] = fma(-x, q[cur][u][0], f[m]);
        if (m + 1 < l) f[m + 1] = fma(-x, q[cur][u][1], f[m + 1]);
      }
      __builtin_amdgcn_sched_barrier(0);
      cur = (cur + 1) % RD;
    }
  }
}

// ------------------------------------------------------------------------------- outer block
// The whole factorisation of the 256 x 256 diagonal block of an outer block in ONE workgroup: its ten 64 x 64
// tiles (upper triangle) are read once and never go back to memory in between.  Eight wavefronts in two groups
// with separate programs (and so separate register allocations: the tiles fill most of the registers of the
// first group, a factorisation those of a wavefront of the second); both run the same number of barriers.
// After the factorisation of tile (3, 3), for K = 3, 2, 1 (inner blocks):
//   wavefronts 4 .. 4+K-1 solve for the panels V_iK, one tile each, wavefront 7 inverts V_KK;        | barrier
//   wavefronts 0-3 store the V_iK, update tile (K-1, K-1) (F_ij -= V_iK V_jK^T, mm64_sub; they hold
//   the tiles (i <= j < K) in registers) and put it into T;                                          | barrier
//   wavefront 4 factors tile (K-1, K-1) WHILE wavefronts 0-3 update the other tiles;                 | barrier
//   wavefronts 0-3 move the rest of tile column K-1 to the LDS slots.                                | barrier
// and at the end wavefront 7 inverts V_00.  Outputs: V_iK to Vob (for tall_kernel and trinv_kernel), Winv_K to Dinv.
// Tiles past the end of the matrix are identity / zero padding and are carried along (only the last outer block of
// a ragged n has any).
constexpr int OBF_LDS = (DIAG_LDS_DOUBLES + 3 * NB * LDT) * 8;
struct ObfShared { double *T, *colb, *dsh, *slot0; };

__device__ __forceinline__ void obf_invert(const Sweep& a, const ObfShared& sh, int kb, int nbi) {
  if (kb >= nbi) return;                                      // (a padding tile: nothing to store)
  const int lane = threadIdx.x & 63;
  double wv[NB];
  inverse_wave(sh.T, sh.dsh, wv);
  double* D = a.Dinv + (int64_t)(a.jlo + kb) * NB * NB;
#pragma unroll
  for (int cc = 0; cc < NB; ++cc) D[lane * NB + cc] = wv[cc];
}

template <int KB>
__device__ __forceinline__ void obf_seq_step(const Sweep& a, const ObfShared& sh, int nbi) {
  const int w = (threadIdx.x >> 6) - 4;
  if (w == 3) obf_invert(a, sh, KB, nbi);
  if (w < KB) solve_wave(sh.T, sh.dsh, sh.slot0 + w * NB * LDT);
  __syncthreads();                                            // the panels are in the slots; T and dsh are free
  __syncthreads();                                            // tile (KB-1, KB-1) is in T
  if (w == 0) cholesky_wave(a, sh.T, sh.colb, sh.dsh, (a.jlo + KB - 1) * NB);
  __syncthreads();                                            // its factor is in T; the slots are free
  __syncthreads();                                            // the next panels' tiles are in the slots
}

template <int KB>
__device__ __forceinline__ void obf_mm_step(const Sweep& a, const ObfShared& sh, double (&tg)[6][4][4]) {
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int c = threadIdx.x & 63, rb = threadIdx.x >> 6;
  auto slot = [&](int i) { return sh.slot0 + i * NB * LDT; };
  constexpr int DIAG = (KB - 1) * KB / 2 + KB - 1;            // tile (KB-1, KB-1)
  __syncthreads();
#pragma unroll
  for (int i = 0; i < KB; ++i)
#pragma unroll
    for (int p = 0; p < 16; ++p)
      a.Vob[(int64_t)(i * NB + rb + 4 * p) * NBO + KB * NB + c] = slot(i)[c * LDT + rb + 4 * p];
  // the tile the next factorisation waits for first
  mm64_sub(slot(KB - 1), slot(KB - 1), tg[DIAG]);             // A[r][l] = V_iK[r][l], B[l][cc] = V_jK[cc][l]
#pragma unroll
  for (int p = 0; p < 4; ++p)
#pragma unroll
    for (int q = 0; q < 4; ++q) sh.T[(4 * ty + p) * LDT + mm_col(tx, q)] = tg[DIAG][p][q];
  __syncthreads();
#pragma unroll
  for (int j = 0; j < KB; ++j)
#pragma unroll
    for (int i = 0; i <= j; ++i)
      if (j * (j + 1) / 2 + i != DIAG) mm64_sub(slot(i), slot(j), tg[j * (j + 1) / 2 + i]);
  __syncthreads();                                            // everyone is done with the slots
#pragma unroll
  for (int i = 0; i < KB - 1; ++i)
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) slot(i)[(4 * ty + p) * LDT + mm_col(tx, q)] = tg[(KB - 1) * KB / 2 + i][p][q];
  __syncthreads();
}

__global__ __launch_bounds__(512) void ob_factor_kernel(Sweep a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  ObfShared sh;
  sh.T = reinterpret_cast<double*>(smem_raw);
  sh.colb = sh.T + NB * LDV;
  sh.dsh = sh.colb + 2 * NB;
  sh.slot0 = sh.dsh + NB;
  const int nbi = (a.o1 - a.o0 + NB - 1) / NB;
  auto at = [&](int row, int col) {                           // identity where the matrix ends
    return (row < a.n && col < a.n) ? a.F[(int64_t)row * a.ldf + col] : (row == col ? 1.0 : 0.0);
  };
  if (threadIdx.x < 256) {
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
    // tile (i, j), i <= j < 3, lives in tg[j * (j + 1) / 2 + i], thread (ty, tx) holding rows 4 ty + p, columns mm_col(tx, q)
    double tg[6][4][4];
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
      for (int i = 0; i <= j; ++i)
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            tg[j * (j + 1) / 2 + i][p][q] = at(a.o0 + i * NB + 4 * ty + p, a.o0 + j * NB + mm_col(tx, q));
    __syncthreads();                                          // tile column 3 is in LDS
    __syncthreads();                                          // tile (3, 3) is factored
    obf_mm_step<3>(a, sh, tg);
    obf_mm_step<2>(a, sh, tg);
    obf_mm_step<1>(a, sh, tg);
  } else {
    const int c = threadIdx.x & 63, w = (threadIdx.x >> 6) - 4;
    // column 3 of the tiles: (3, 3) to T, the others to the slots, row-major
    double ld[4][16];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int p = 0; p < 16; ++p) ld[i][p] = at(a.o0 + i * NB + w + 4 * p, a.o0 + 3 * NB + c);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      double* dst = i < 3 ? sh.slot0 + i * NB * LDT : sh.T;
#pragma unroll
      for (int p = 0; p < 16; ++p) dst[(w + 4 * p) * LDT + c] = ld[i][p];
    }
    __syncthreads();
    if (w == 0) cholesky_wave(a, sh.T, sh.colb, sh.dsh, (a.jlo + 3) * NB);
    __syncthreads();
    obf_seq_step<3>(a, sh, nbi);
    obf_seq_step<2>(a, sh, nbi);
    obf_seq_step<1>(a, sh, nbi);
    if (w == 3) obf_invert(a, sh, 0, nbi);
  }
}

// ------------------------------------------------------------------------------- tall
// The rows above the outer block: for a 64-row tile i, from the last inner block K of OB to the first,
// V_iK = F_iK Winv_K^T (stored in place) and F_ij -= V_iK V_jK^T for the tiles j of OB left of K, with the
// V_jK of OB's own rows from Vob.  The four F_i,* tiles stay in registers between the steps; the ten products
// form a chain, so the right operand of the next one (known in advance) is fetched into registers while the
// current one runs and goes to the other of two LDS buffers.  grid: jlo workgroups.
constexpr int TALL_LDS = 3 * NB * LDT * 8;
__global__ __launch_bounds__(256) void tall_kernel(Sweep a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  double* As = reinterpret_cast<double*>(smem_raw);
  double* Bs0 = As + NB * LDT;
  const int r0 = blockIdx.x * NB, nbi = (a.o1 - a.o0 + NB - 1) / NB;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int c = threadIdx.x & 63, rb = threadIdx.x >> 6;
  // right operands in the order of use: for K = nbi-1 .. 0: Winv_K, then V_jK for j = K-1 .. 0
  double nxt[16];
  auto fetch = [&](int kl, int j) {                       // j < 0: Winv_kl
    const double* src = j < 0 ? a.Dinv + (int64_t)(a.jlo + kl) * NB * NB : a.Vob + (int64_t)j * NB * NBO + kl * NB;
    const int ld = j < 0 ? NB : NBO;
#pragma unroll
    for (int p = 0; p < 16; ++p) nxt[p] = src[(int64_t)(rb + 4 * p) * ld + c];
  };
  auto put_b = [&](double* Bs) {                          // B[l][cc] = src[cc][l]
#pragma unroll
    for (int p = 0; p < 16; ++p) Bs[c * LDT + rb + 4 * p] = nxt[p];
  };
  fetch(nbi - 1, -1);
  double f[4][4][4];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = a.o0 + b * NB + mm_col(tx, q);
        f[b][p][q] = (b < nbi && col < a.n) ? a.F[(int64_t)(r0 + 4 * ty + p) * a.ldf + col] : 0.0;
      }
  int flip = 0;
#pragma unroll
  for (int kl = 3; kl >= 0; --kl) {
    if (kl >= nbi) continue;
    // (the barrier at the end of the product before this one has retired As and the buffer written now)
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) As[(mm_col(tx, q)) * LDT + 4 * ty + p] = f[kl][p][q];
    double* Bs = Bs0 + flip * NB * LDT;
    flip ^= 1;
    put_b(Bs);
    if (kl > 0) fetch(kl, kl - 1);
    __syncthreads();
    double v[4][4];
    mm64(As, Bs, v);
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = a.o0 + kl * NB + mm_col(tx, q);
        if (col < a.n) a.F[(int64_t)(r0 + 4 * ty + p) * a.ldf + col] = v[p][q];
      }
    if (kl == 0) break;
    __syncthreads();                                      // everyone has read As
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) As[(mm_col(tx, q)) * LDT + 4 * ty + p] = v[p][q];
#pragma unroll
    for (int j = 2; j >= 0; --j) {
      if (j >= kl) continue;
      double* Bj = Bs0 + flip * NB * LDT;
      flip ^= 1;
      put_b(Bj);
      if (j > 0) fetch(kl, j - 1); else fetch(kl - 1, -1);
      __syncthreads();
      double acc[4][4];
      mm64(As, Bj, acc);
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) f[j][p][q] -= acc[p][q];
    }
    __syncthreads();                                      // everyone has read As before the next panel overwrites it
  }
}

// ------------------------------------------------------------------------------ trinv
// U_OB,OB = V_OB,OB^-1 from the inner blocks: U_ll = Winv_l and, for k < l,
// U_kl = -Winv_k sum_{k < j <= l} V_kj U_jl.  One workgroup per block column l; results go to the
// dense scratch Uob (ld 256, zeros below the diagonal), from which they are copied into F afterwards
// (the other workgroups still read F's block while this one runs).
// The steps of a block column form a chain of 64^3 products, so what counts is the latency of a step:
// the finished blocks U_jl stay in LDS (slot j; they are the right operands of all later steps), and the
// left operand of the next product (V_kj or Winv_k, known in advance) is fetched into registers while
// the current product runs.
constexpr int TRINV_LDS = 4 * NB * LDT * 8;      // the staged left operand + slots 1..3
__global__ __launch_bounds__(256) void trinv_kernel(Sweep a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  double* As = reinterpret_cast<double*>(smem_raw);
  auto slot = [&](int j) { return As + j * NB * LDT; };           // j = 1..3
  const int l = blockIdx.x, kb0 = a.o0 / NB, wo = a.o1 - a.o0;
  const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
  const int nbi = (wo + NB - 1) / NB;
  // blocks below the diagonal of this block column are zero
  for (int k = l + 1; k < nbi; ++k)
    for (int idx = threadIdx.x; idx < NB * NB; idx += 256) a.Uob[(int64_t)(k * NB + (idx >> 6)) * 256 + l * NB + (idx & 63)] = 0.0;
  auto put_global = [&](int k, const double (&v)[4][4]) {
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) a.Uob[(int64_t)(k * NB + 4 * ty + p) * 256 + l * NB + mm_col(tx, q)] = v[p][q];
  };
  auto put_slot = [&](double* dst, const double (&v)[4][4], double sign) {    // right-operand layout: dst[m * LDT + c]
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) dst[(4 * ty + p) * LDT + mm_col(tx, q)] = sign * v[p][q];
  };
  double acc[4][4];
  {
    const double* D = a.Dinv + (int64_t)(kb0 + l) * NB * NB;
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[p][q] = D[(4 * ty + p) * NB + mm_col(tx, q)];
  }
  put_global(l, acc);
  if (l == 0) return;
  put_slot(slot(l), acc, 1.0);

  // the left operands in the order they are used: for k = l-1 .. 0: V_k,k+1 .. V_k,l, then Winv_k
  const int c = threadIdx.x & 63, rb = threadIdx.x >> 6;
  double nxt[16];
  auto fetch = [&](int t) {
    int k = l - 1, j = -1;
    bool found = false;
    for (; k >= 0; --k) {
      const int cnt = l - k + 1;
      if (t < cnt) { j = t < l - k ? k + 1 + t : -1; found = true; break; }
      t -= cnt;
    }
    if (!found) return;
    const double* src = j >= 0 ? a.Vob : a.Dinv + (int64_t)(kb0 + k) * NB * NB;
    const int64_t ld = j >= 0 ? NBO : NB;
    const int r0 = j >= 0 ? k * NB : 0, c0 = j >= 0 ? j * NB : 0, lim = j >= 0 ? NBO : NB;
#pragma unroll
    for (int p = 0; p < 16; ++p) {
      const int r = rb + 4 * p;
      nxt[p] = (r0 + r < lim && c0 + c < lim) ? src[(int64_t)(r0 + r) * ld + c0 + c] : 0.0;
    }
  };
  auto stage_next = [&]() {                       // left-operand layout: As[m * LDT + i] = A[i][m]
#pragma unroll
    for (int p = 0; p < 16; ++p) As[c * LDT + rb + 4 * p] = nxt[p];
  };
  int t = 0;
  fetch(t++);
  for (int k = l - 1; k >= 0; --k) {
    double sum[4][4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) sum[p][q] = 0.0;
    for (int j = k + 1; j <= l; ++j) {
      __syncthreads();                            // the product before is done with As; slot writes are visible
      stage_next();
      fetch(t++);
      __syncthreads();
      mm64(As, slot(j), acc);
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) sum[p][q] += acc[p][q];
    }
    // U_kl = Winv_k (-sum); -sum goes where U_kl will live (for k = 0, which no later step reads, into
    // slot l, whose block has just been used for the last time)
    double* tmp = k >= 1 ? slot(k) : slot(l);
    __syncthreads();
    stage_next();
    fetch(t++);
    put_slot(tmp, sum, -1.0);
    __syncthreads();
    mm64(As, tmp, acc);
    put_global(k, acc);
    if (k >= 1) {
      __syncthreads();                            // everyone has read -sum
      put_slot(tmp, acc, 1.0);
    }
  }
}

// dst[r][c] = src[r][c] for an (rows x cols) block of doubles; `upper`: only c >= r is copied.
__global__ void copy_block_kernel(const double* src, int64_t lds_, double* dst, int64_t ldd, int rows, int cols,
                                  int upper) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x, r = blockIdx.y;
  if (c >= cols || r >= rows || (upper && c < r)) return;
  dst[(int64_t)r * ldd + c] = src[(int64_t)r * lds_ + c];
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

// bf16 hi/lo split of the strictly upper triangle of an fp32 matrix (rows flagged in `zero_rows` read as 0), padded
// to np x np; entries on and below the diagonal are not read and come out as 0.  Both uses want exactly that: Eq. 17
// masks dXXT L to its strictly upper part and L is lower triangular, so entry (i, k) of dXXT only ever meets a
// non-zero of L when k > i, and the masked product itself is strictly upper.
// `info` (may be NULL): a NaN or Inf among the entries read is reported as info[0] = -(1 + row of the entry).
__global__ __launch_bounds__(256) void split_rows_kernel(const float* A, int64_t lda, int n, const uint8_t* zero_rows,
                                                         uint16_t* Ah, uint16_t* Al, int64_t np, int32_t* info) {
  const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x, r = blockIdx.y;
  if (c >= np) return;
  float v = 0.f;
  if (r < n && c < n && c > r && !(zero_rows && zero_rows[r])) v = A[r * lda + c];
  if (info && !__builtin_isfinite(v)) atomicMin(info, -(1 + (int)r));
  const uint16_t h = bf16_rne(v);
  Ah[r * np + c] = h;
  Al[r * np + c] = bf16_rne(v - bf16_f32(h));
}

}  // namespace gptaq

using namespace gptaq;

namespace {
struct PrepLayout {
  int64_t np;
  int64_t rp;                      // rows of a sliced operand that spans the whole matrix
  size_t off_F, off_Dinv, off_lam, off_dead, off_O, off_b[6], off_Uob, off_Vob, off_pl[5], off_sc[5], total;
};
PrepLayout prep_layout(int64_t n) {
  PrepLayout L;
  const int tile = gemm_tile_for(n, n);
  L.np = round_up(n, tile);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o += (bytes + 255) / 256 * 256; return r; };
  L.off_lam = take(256);
  L.off_F = take((size_t)n * round_up(n, 16) * 8);
  L.off_Dinv = take((size_t)round_up(n, NB) * NB * 8);
  L.off_dead = take((size_t)n);
  L.off_O = take((size_t)L.np * L.np * 4);
  for (int i = 0; i < 6; ++i) L.off_b[i] = take((size_t)L.np * L.np * 2);
  L.off_Uob = take((size_t)NBO * NBO * 8);
  L.off_Vob = take((size_t)3 * NBO * NBO * 8);      // three in turn: the inverse chain reads a block's while the next two are written
  // sliced operands of the rank-256 products: V_I,OB (two: the helper stream reads one while the next is
  // written), R_OB,J / U_OB,J, and U_OB,OB by rows and by columns
  L.rp = round_up(n, 128);
  for (int i = 0; i < 5; ++i) {
    const int64_t rows = i < 3 ? L.rp : NBO;
    L.off_pl[i] = take(I8Operand::plane_bytes(rows));
    L.off_sc[i] = take((size_t)rows * 4);
  }
  L.total = o;
  return L;
}

}  // namespace

extern "C" size_t gptaq_prepare_workspace_bytes(int64_t n) {
  if (n <= 0) return 0;
  return prep_layout(n).total;
}

extern "C" int gptaq_prepare(float* H, float* dXXT, int64_t n, int64_t ldh, float damp, uint8_t* dead,
                             int32_t* info, void* ws, size_t ws_bytes, void* stream) {
  if (!H || !dXXT || !info || !ws) return GPTAQ_ENULL;
  // (several kernels put a row index in gridDim.y, which ends at 65535: rows of the padded n x n buffers)
  if (n <= 0 || ldh < n || n > 65280 || !(damp >= 0.f)) return GPTAQ_EDIM;
  if ((uintptr_t)ws & 255) return GPTAQ_EWORKSPACE;
  const PrepLayout L = prep_layout(n);
  if (ws_bytes < L.total) return GPTAQ_EWORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  {
    static LdsLimitOnce once_obf, once_tall, once_trinv;
    hipError_t e = once_obf.ensure((const void*)&ob_factor_kernel, OBF_LDS);
    if (e == hipSuccess) e = once_tall.ensure((const void*)&tall_kernel, TALL_LDS);
    if (e == hipSuccess) e = once_trinv.ensure((const void*)&trinv_kernel, TRINV_LDS);
    if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
  }
  unsigned char* base = (unsigned char*)ws;
  double* lam = (double*)(base + L.off_lam);
  double* F = (double*)(base + L.off_F);
  double* Dinv = (double*)(base + L.off_Dinv);
  uint8_t* deadbuf = dead ? dead : (uint8_t*)(base + L.off_dead);
  float* Obuf = (float*)(base + L.off_O);
  I8Operand sl[5];
  for (int i = 0; i < 5; ++i) sl[i] = I8Operand{base + L.off_pl[i], (int32_t*)(base + L.off_sc[i]), i < 3 ? L.rp : (int64_t)NBO};
  const I8Operand &RJs = sl[2], &Urow = sl[3], &Ucol = sl[4];
  const int64_t ldf = round_up(n, 16);
  double* Uob = (double*)(base + L.off_Uob);
  double* Vob3 = (double*)(base + L.off_Vob);
  uint16_t* bb[6];
  for (int i = 0; i < 6; ++i) bb[i] = (uint16_t*)(base + L.off_b[i]);
  const int ni = (int)n;

  hipLaunchKernelGGL(diag_stats_kernel, dim3(1), dim3(1024), 0, s, H, ldh, ni, damp, deadbuf, lam, info);
  GPTAQ_LAUNCH_CHECK();
  hipLaunchKernelGGL(build_F_kernel, dim3((unsigned)((n + 255) / 256), (unsigned)n), dim3(256), 0, s, H, ldh, ni,
                     lam, F, ldf, info);
  GPTAQ_LAUNCH_CHECK();

  // The sweep is two chains of kernels over the outer blocks OB = nob-1 .. 0 (I: rows above, J: columns right):
  //   factor chain (caller's stream): inner factorisation of block column OB, int8 digits of V_I,OB, Schur update
  //                                   of the next block column;
  //   inverse chain (helper stream):  Schur update of the rest of F_II, U_OB,OB, then U_OB,J = U_OB,OB R_OB,J, R_I,J -= V_I,OB U_OB,J, R_I,OB = -V_I,OB U_OB,OB.
  // The rank-256 products run on the int8 matrix cores from digit-sliced operands (gemm_i8s.hip).
  // The inverse chain of a block needs that block's V_I,OB digits and diagonal inverses and nothing later from the
  // factor chain, and it only writes columns >= o0 of F while the factor chain has moved on to columns < o0,
  // so the two overlap: the small sequential kernels of one hide behind the rank-256 products of the other.
  // The V_I,OB digits alternate between two buffers; an event per block and direction orders the streams.
  std::lock_guard<std::mutex> side_lock(side_stream_mutex());
  const int nob = (int)((n + NBO - 1) / NBO);
  SideStream* side = side_stream(3 * nob + 2);
  if (!side) { set_last_hip_error(hipGetLastError()); return GPTAQ_ELAUNCH; }
  hipStream_t sb = side->stream;
  {
    ProfScope sweep_scope(kProfFactor, s);
    Sweep a;
    a.F = F; a.ldf = ldf; a.n = ni; a.nblk = (int)((n + NB - 1) / NB); a.Dinv = Dinv; a.info = info; a.Uob = Uob;
    bool ok = true;
    auto chk = [&](hipError_t e) { if (e != hipSuccess && ok) { ok = false; set_last_hip_error(e); } };
    auto copy = [&](hipStream_t st, const double* src, int64_t lds_, double* dst, int64_t ldd, int rows, int cols, int upper) {
      if (rows <= 0 || cols <= 0) return;
      hipLaunchKernelGGL(copy_block_kernel, dim3((cols + 255) / 256, rows), dim3(256), 0, st, src, lds_, dst, ldd, rows,
                         cols, upper);
    };
    hipEvent_t ev_fork = side->events[3 * nob];
    chk(hipEventRecord(ev_fork, s));                          // the helper stream starts behind build_F
    chk(hipStreamWaitEvent(sb, ev_fork, 0));
    for (int ob = nob - 1; ob >= 0 && ok; --ob) {
      const int o0 = ob * NBO, o1 = (int)(n < o0 + NBO ? n : o0 + NBO), wo = o1 - o0;
      const I8Operand& Vs = sl[ob & 1];
      hipEvent_t ev_factored = side->events[2 * ob], ev_inverted = side->events[2 * ob + 1];
      a.o0 = o0; a.o1 = o1; a.jlo = o0 / NB;
      // ---- factor chain
      // (the inverse chain of block ob + 3, the last reader of this Vob, was waited for before block ob + 1's slices)
      a.Vob = Vob3 + (size_t)(ob % 3) * NBO * NBO;
      hipLaunchKernelGGL(ob_factor_kernel, dim3(1), dim3(512), OBF_LDS, s, a);
      if (a.jlo > 0) hipLaunchKernelGGL(tall_kernel, dim3(a.jlo), dim3(256), TALL_LDS, s, a);
      // this buffer of V_I,OB digits was last read by the inverse chain of block ob + 2
      if (ob + 2 <= nob - 1) chk(hipStreamWaitEvent(s, side->events[2 * (ob + 2) + 1], 0));
      chk(launch_slice_i8(F + o0, ldf, 1, o0, wo, Vs, s));     // V_I,OB, the operand of all four products with it
      chk(hipEventRecord(ev_factored, s));
      // Schur complement of everything above/left of the outer block, F_II -= V_I,OB V_I,OB^T, in two parts:
      // the block column the next outer block factors (here, it is on the critical path) and the rest (upper
      // tiles, on the helper stream).  The next block's part-one update overlaps this block's part two in
      // memory, so it waits for it.
      const int c_lo = o0 > NBO ? o0 - NBO : 0;
      if (ob + 1 <= nob - 1) chk(hipStreamWaitEvent(s, side->events[2 * nob + ob + 1], 0));
      chk(launch_gemm_i8s(Vs, 0, Vs, c_lo, F + c_lo, ldf, o0, o0 - c_lo, wo, -1.0, 1, 0, s));
      // ---- inverse chain
      chk(hipStreamWaitEvent(sb, ev_factored, 0));
      chk(launch_gemm_i8s(Vs, 0, Vs, 0, F, ldf, c_lo, c_lo, wo, -1.0, 1, 1, sb));
      chk(hipEventRecord(side->events[2 * nob + ob], sb));
      double* FJ = F + (int64_t)o0 * ldf + o1;                  // block row OB right of the diagonal block
      chk(launch_slice_i8(FJ, 1, ldf, ni - o1, wo, RJs, sb));   // R_OB,J (digits per column of it)
      hipLaunchKernelGGL(trinv_kernel, dim3((wo + NB - 1) / NB), dim3(256), TRINV_LDS, sb, a);
      copy(sb, Uob, 256, F + (int64_t)o0 * ldf + o0, ldf, wo, wo, 1);         // U_OB,OB into F
      chk(launch_slice_i8(Uob, 256, 1, wo, wo, Urow, sb));
      chk(launch_slice_i8(Uob, 1, 256, wo, wo, Ucol, sb));
      chk(launch_gemm_i8s(Urow, 0, RJs, 0, FJ, ldf, wo, ni - o1, wo, 1.0, 0, 0, sb));           // U_OB,J = U_OB,OB R_OB,J
      chk(launch_slice_i8(FJ, 1, ldf, ni - o1, wo, RJs, sb));                                    // now U_OB,J
      chk(launch_gemm_i8s(Vs, 0, RJs, 0, F + o1, ldf, o0, ni - o1, wo, -1.0, 1, 0, sb));         // R_I,J -= V_I,OB U_OB,J
      chk(launch_gemm_i8s(Vs, 0, Ucol, 0, F + o0, ldf, o0, wo, wo, -1.0, 0, 0, sb));             // R_I,OB = -V_I,OB U_OB,OB
      chk(hipGetLastError());
      chk(hipEventRecord(ev_inverted, sb));
    }
    // join: everything after the sweep runs on the caller's stream (blocks 0 and 1 have not been waited for yet)
    if (ok) {
      chk(hipStreamWaitEvent(s, side->events[1], 0));
      if (nob > 1) chk(hipStreamWaitEvent(s, side->events[3], 0));
    }
    if (!ok) {
      // a launch or an event call failed part-way: whatever the helper stream was given so far must still be behind
      // the caller's stream when the call returns, so the join is made with a fresh record of the helper stream
      const hipError_t keep = (hipError_t)gptaq_last_hip_error();
      if (hipEventRecord(ev_fork, sb) == hipSuccess) hipStreamWaitEvent(s, ev_fork, 0);
      set_last_hip_error(keep);
      return GPTAQ_ELAUNCH;
    }
  }
  // U -> H (fp32) and the bf16 splits; dXXT (dead rows zeroed) split.
  const int64_t np = L.np;
  uint16_t *Uh = bb[0], *Ul = bb[1], *Uth = bb[2], *Utl = bb[3], *Ah = bb[4], *Al = bb[5];
  hipLaunchKernelGGL(extract_U_kernel, dim3((unsigned)(np / 64), (unsigned)(np / 64)), dim3(256), 0, s, F, ldf, ni, H,
                     ldh, Uh, Ul, Uth, Utl, np);
  GPTAQ_LAUNCH_CHECK();
  hipLaunchKernelGGL(split_rows_kernel, dim3((unsigned)((np + 255) / 256), (unsigned)np), dim3(256), 0, s, dXXT, ldh,
                     ni, deadbuf, Ah, Al, np, info);
  GPTAQ_LAUNCH_CHECK();

  // The K ranges of these two products are triangular, so tiles differ in length by the whole of K: the tile list is
  // dealt to the XCDs four tiles at a time (`deal`), not in contiguous runs (n = 11008: 2.8 -> 1.2 ms per product), and
  // while 256-tiles make a single round, the longest one sets the time and 128-tiles balance better (n = 4096)
  const int t256 = gemm_tile_for(n, n);
  const int tile = (t256 == 256 && (np / 256) * (np / 256) <= 256) ? 128 : t256;
  GemmBatch b{};
  b.nprob = 1; b.tile = tile;
  GemmProblem& g = b.p[0];
  // O = triu(dXXT U^T, 1): O[i][a] = sum_{b >= a} dXXT[i][b] U[a][b]
  g.C = Obuf; g.ldc = np; g.M = ni; g.N = ni; g.K = (int)np;
  g.tiles_m = g.tiles_n = (int)(np / tile);
  g.kind = 2; g.nterm = 1; g.tile_mode = 1; g.k_mode = 1; g.store_mode = 2; g.deal = 1;
  g.term[0] = {{Ah, Al}, {Uh, Ul}, np, np, 32, 32};
  hipError_t e;
  {
    ProfScope ps(kProfPGemm, s);
    e = launch_gemm(b, s);
  }
  if (e != hipSuccess) { set_last_hip_error(e); return GPTAQ_ELAUNCH; }
  // split O (reuses the dXXT split buffers), then P = O U: P[i][j] = sum_{i < a <= j} O[i][a] U[a][j]
  hipLaunchKernelGGL(split_rows_kernel, dim3((unsigned)((np + 255) / 256), (unsigned)np), dim3(256), 0, s, Obuf, np,
                     ni, (const uint8_t*)nullptr, Ah, Al, np, (int32_t*)nullptr);
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
