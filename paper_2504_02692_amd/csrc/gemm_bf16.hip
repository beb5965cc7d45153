// bf16 x bf16 -> fp32 MFMA GEMM for gfx950:  C (+)= sum over terms of (sum of cross products) L R^T.
//
// Every dense contraction of the solve goes through this kernel (Algorithm 1 line 2: H and
// dXXT; line 4: the two products of Theorem 4.2; lines 11-12: the lazy trailing update of
// Eq. 18).  Where fp32 operands need more than bf16's 8 bits, an operand is split into bf16
// hi + lo (about 2^-17 relative) and the cross products hi*hi + hi*lo + lo*hi are summed in fp32.
//
// Tiling: a 256-thread workgroup owns a BT x BT tile of C (BT = 256 or 128); its four
// wavefronts sit 2 x 2 and each accumulates a (BT/2)^2 sub-tile with
// v_mfma_f32_32x32x16_bf16 (accumulators in AGPRs).  Operand k-tiles (BT rows x 32 bf16) go
// from global memory straight into LDS (global_load_lds_dwordx4, no VGPR staging) through a
// ring of LDS stages, ahead of the multiply; fragment reads are ds_read_b128 on an
// XOR-swizzled layout and run one k-step ahead of the MFMAs.
//
// Feeding the operands is what bounds this kernel: a CU takes at most ~22 bytes per clock from its L2
// into LDS (measured; less when lines come from HBM), which is about what one 256 x 256 product per
// two operand tiles needs at full MFMA rate.  So operand tiles are shared between cross products: per
// k-tile a term loads its NL left and NR right operand tiles once and multiplies all listed
// (left, right) pairs from them - dXXT's hi and lo halves share the X tile, and the three products of
// a split term need four tiles instead of six.  The loads of a k-tile are issued one by one between
// the MFMAs of an earlier k-tile, and the barriers carry no memory fence, so that loads stay in
// flight across them (see wg_barrier).
#include "common.h"

namespace gptaq {

template <int KIND> struct KindTraits;
template <> struct KindTraits<0> { static constexpr int NL = 1, NR = 1, NPAIR = 1, NSTAGE = 4; };
template <> struct KindTraits<1> { static constexpr int NL = 2, NR = 1, NPAIR = 2, NSTAGE = 3; };
template <> struct KindTraits<2> { static constexpr int NL = 2, NR = 2, NPAIR = 3, NSTAGE = 2; };
// pair p of a kind: (left index, right index)
__device__ __forceinline__ constexpr int pair_l(int kind, int p) { return kind == 0 ? 0 : kind == 1 ? p : (p == 2 ? 1 : 0); }
__device__ __forceinline__ constexpr int pair_r(int kind, int p) { return kind == 2 ? (p == 1 ? 1 : 0) : 0; }

// Workgroup barrier without the memory fence of __syncthreads(): that fence makes the compiler drain
// every outstanding global -> LDS load (vmcnt(0)) at each barrier, which would cut the load pipeline
// down to one k-tile.  The waits a barrier needs here are written out by hand before it.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int N> __device__ __forceinline__ void wait_vm_and_lds() {
  // vmcnt <= N (vmcnt is split over bits 3:0 and 15:14), lgkmcnt == 0, expcnt untouched
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4));
}

constexpr int kLds256 = 3 * 3 * 256 * 64;    // largest ring: 3 stages x 3 operand tiles (2 x 4 and 4 x 2 are smaller)
constexpr int kLds128 = 3 * 3 * 128 * 64;

template <int BT, int KIND, bool MULTI>
__device__ __forceinline__ void tile_loop(const GemmProblem& P, unsigned char* smem, int m0, int n0, int klo, int nk,
                                          f32x16 (&acc)[BT / 64][BT / 64]) {
  using T = KindTraits<KIND>;
  constexpr int NL = T::NL, NR = T::NR, NOP = NL + NR, NSTAGE = T::NSTAGE;
  constexpr int WT = BT / 2, FR = WT / 32;
  constexpr int OPB = BT * 64;           // bytes of one operand k-tile (BT rows x 32 bf16)
  constexpr int STAGE_BYTES = NOP * OPB;
  constexpr int LPW = BT / 64;           // 1 KB wave-loads per operand per wave per k-tile
  constexpr int TL = NOP * LPW;          // loads per k-tile per wave
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int total_it = nk * P.nterm;

  // ---- LDS tile format.  An operand k-tile is BT rows x 32 bf16 (64 B per row).  The LDS of gfx950
  // has 64 banks (256 B per clock), and a ds_read_b128 serves 16 lanes per clock, so 16 consecutive
  // fragment rows of one 16-byte chunk column must land in 16 different 16-byte slots of a 256-byte
  // line.  Four rows share a line; slot = (row & 3) * 4 + (chunk ^ (line & 3)): the four lines that
  // 16 consecutive rows touch use four different XOR values, i.e. disjoint slot sets.
  // Loads go global -> LDS directly: lane l of a wave writes the 16 bytes at LDS base + 16 l, so a
  // wave fills 4 consecutive lines (16 rows) and each lane fetches the (row, chunk) of its slot.
  const int ld_line = lane >> 4;
  const int ld_row = ld_line * 4 + ((lane & 15) >> 2);
  const int ld_chunk = (lane & 3) ^ ld_line;
  // The TL wave loads of a k-tile are issued one at a time, spread between the MFMAs of the k-tile
  // before it (a wave stalls ~50 clocks per 1 KB load it hands to the memory pipeline; in a burst that
  // is time the matrix unit idles).  Past the last k-tile the last one is fetched again into the stage
  // that has just been retired, which keeps the loop and its wait counts free of special cases.
  // The tiles are loaded in order, so the source is a cursor: per-lane pointers to the next tile, moved on
  // by one k-tile after each (recomputed only where the second term starts).
  struct TileSrc {
    const uint16_t* l[NL];
    const uint16_t* r[NR];
    int64_t lstep, rstep;     // 16 rows, in elements
    int64_t lkt, rkt;         // one k-tile, in elements
    unsigned char* st;        // this wave's part of the stage the tile goes to
    int seq;                  // number of the tile in load order (not clamped)
  };
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  auto seek_term = [&](TileSrc& c, int t) {
    const GemmTerm& tm = P.term[t];
    const int64_t kt = klo / kGemmBK;
    const int64_t lo = (int64_t)(m0 + wave * LPW * 16 + ld_row) * tm.ldl + kt * tm.ktl + ld_chunk * 8;
    const int64_t ro = (int64_t)(n0 + wave * LPW * 16 + ld_row) * tm.ldr + kt * tm.ktr + ld_chunk * 8;
#pragma unroll
    for (int o = 0; o < NL; ++o) c.l[o] = tm.L[o] + lo;
#pragma unroll
    for (int o = 0; o < NR; ++o) c.r[o] = tm.R[o] + ro;
    c.lstep = 16 * tm.ldl;
    c.rstep = 16 * tm.ldr;
    c.lkt = tm.ktl;
    c.rkt = tm.ktr;
  };
  // moves the cursor on by one k-tile; `stage` (static) is the stage the new tile goes to
  auto next_tile = [&](TileSrc& c, int stage) {
    ++c.seq;
    c.st = smem + stage * STAGE_BYTES + wave_s * LPW * 1024;
    if (MULTI && c.seq == nk && c.seq < total_it) {
      seek_term(c, 1);
    } else {
      const int64_t ls = c.seq < total_it ? c.lkt : 0, rs = c.seq < total_it ? c.rkt : 0;
#pragma unroll
      for (int o = 0; o < NL; ++o) c.l[o] += ls;
#pragma unroll
      for (int o = 0; o < NR; ++o) c.r[o] += rs;
    }
  };
  // q-th load of the tile: q = j * NOP + o (16-row slab j of operand o)
  auto load_one = [&](const TileSrc& c, int q) {
    const int j = q / NOP, o = q % NOP;
    const uint16_t* src = o < NL ? c.l[o < NL ? o : 0] + j * c.lstep : c.r[o < NL ? 0 : o - NL] + j * c.rstep;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(c.st + j * 1024 + o * OPB), 16, 0, 0);
  };

  // fragment reads: lane -> row (lane & 31) of a 32-row block, chunk 2 kk + (lane >> 5)
  const int rl = lane & 31, half = lane >> 5;
  const int fr_line = rl >> 2, fr_x = fr_line & 3, fr_hi = (rl & 3) << 2;
  bf16x8 af[2][NL][FR], bfr[2][NR][FR];
  constexpr int NFRAG = NOP * FR;      // fragments per k-step: NL * FR left, then NR * FR right
  struct FragSrc { const unsigned char* lb; const unsigned char* rb; };
  auto frag_src = [&](int stage, int kk) {
    const int off = (fr_hi | ((kk * 2 + half) ^ fr_x)) << 4;
    FragSrc f;
    f.lb = smem + stage * STAGE_BYTES + (wm * (WT / 4) + fr_line) * 256 + off;
    f.rb = smem + stage * STAGE_BYTES + NL * OPB + (wn * (WT / 4) + fr_line) * 256 + off;
    return f;
  };
  auto read_one = [&](const FragSrc& f, int set, int r) {
    if (r < NL * FR) {
      const int o = r / FR, i = r % FR;
      af[set][o][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(f.lb + o * OPB + i * 8 * 256));
    } else {
      const int o = (r - NL * FR) / FR, i = (r - NL * FR) % FR;
      bfr[set][o][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(f.rb + o * OPB + i * 8 * 256));
    }
  };
  // The MFMAs of one k-step on fragment set `set`.  Between them, one at a time (so that each is issued
  // in the shadow of a running MFMA instead of holding up the next one): the fragment reads of the other
  // set for the following k-step, and loads q0 .. q1-1 of tile `c`.
  constexpr int NM = T::NPAIR * FR * FR;
  static_assert(TL <= NM && NFRAG <= NM, "at most one load and one fragment read per MFMA");
  auto mfma_step = [&](int set, const FragSrc& f, const TileSrc& c, int q0, int q1) {
#pragma unroll
    for (int p = 0; p < T::NPAIR; ++p)
#pragma unroll
      for (int i = 0; i < FR; ++i)
#pragma unroll
        for (int j = 0; j < FR; ++j) {
          const int m = (p * FR + i) * FR + j, nq = q1 - q0;
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][pair_l(KIND, p)][i], bfr[set][pair_r(KIND, p)][j],
                                                              acc[i][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (m < NFRAG) read_one(f, set ^ 1, m);
          if ((m + 1) * nq / NM > m * nq / NM) load_one(c, q0 + m * nq / NM);
          __builtin_amdgcn_sched_barrier(0);
        }
  };
  // Pipeline: k-tile `it` is multiplied from stage it % NSTAGE.  One barrier per k-tile, in the middle of
  // its MFMAs: it publishes tile it+1 (every wave has waited for its own loads of it: they return in
  // order, so "at most so many outstanding" says which have landed) and retires stage it % NSTAGE, whose
  // last fragments were read before it.  Tile it + NSTAGE goes into that stage: its first HF loads are
  // issued behind the barrier, the rest before the next one, so each has at least a whole k-tile of
  // MFMA time to arrive (half of one with two stages).
  constexpr int HF = NSTAGE >= 3 ? TL / 2 : TL;
  constexpr int PENDING = (NSTAGE - 2) * TL;               // loads of later tiles issued by the barrier
  if (total_it <= 0) return;
  TileSrc c;
  seek_term(c, 0);
  c.seq = 0;
  c.st = smem + wave_s * LPW * 1024;
#pragma unroll
  for (int t = 0; t < NSTAGE - 1; ++t) {
#pragma unroll
    for (int q = 0; q < TL; ++q) load_one(c, q);
    next_tile(c, t + 1);
  }
#pragma unroll
  for (int q = 0; q < HF; ++q) load_one(c, q);
  wait_vm_and_lds<PENDING + HF>();
  wg_barrier();
  {
    const FragSrc f0 = frag_src(0, 0);
#pragma unroll
    for (int r = 0; r < NFRAG; ++r) read_one(f0, 0, r);
  }
  // NSTAGE k-tiles per trip, so that every stage number below is a constant (LDS addresses and DMA targets
  // become immediates and scalars instead of per-iteration vector arithmetic)
  for (int it0 = 0; it0 < total_it; it0 += NSTAGE) {
#pragma unroll
    for (int sg = 0; sg < NSTAGE; ++sg) {
      if (it0 + sg < total_it) {
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(0, frag_src(sg, 1), c, HF, TL);
        __builtin_amdgcn_sched_barrier(0);
        wait_vm_and_lds<PENDING>();
        wg_barrier();
        __builtin_amdgcn_sched_barrier(0);
        next_tile(c, sg);                                   // tile it + NSTAGE goes where tile it was
        // (behind the last k-tile these fragment reads fetch a stale stage and nobody uses them)
        mfma_step(1, frag_src((sg + 1) % NSTAGE, 0), c, 0, HF);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  wait_vm_and_lds<0>();   // the surplus loads past the last k-tile
}

// One BT x BT tile of C: tile number `wid` of the batch (see the numbering below).
template <int BT>
__device__ __forceinline__ void gemm_tile(const GemmBatch& b, unsigned char* smem, int wid) {
  constexpr int WT = BT / 2;             // wave tile edge
  constexpr int FR = WT / 32;            // 32x32 MFMA blocks per wave tile edge

  // ---- which tile.  Workgroups are dealt round-robin to the 8 XCDs; inside each problem, give every
  // XCD one contiguous run of tiles so that they share operand tiles in that XCD's L2, and so that
  // every XCD gets the same share of each problem (the problems differ in K).
  int id = wid;
  int pi = 0;
  int ntile = b.ntiles[0];
  if (id >= ntile) { pi = 1; id -= ntile; ntile = b.ntiles[1]; }
  const GemmProblem& P = b.p[pi];
  if (!P.deal) {
    const int per = ntile >> 3, rem = ntile & 7, xcd = id & 7, loc = id >> 3;
    id = xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
  } else if (id < (ntile & ~31)) {
    // With triangular k ranges a contiguous run per XCD would give one XCD the long tiles and another the short ones.
    // Here every XCD takes four consecutive tiles (the four tile rows of one column of a group) out of each 32, so
    // each gets the same mix of lengths, and the 32 workgroups it runs side by side still share four left tiles.
    const int xcd = id & 7, loc = id >> 3;
    id = (((loc >> 2) << 3) + xcd) * 4 + (loc & 3);
  }
  int tm, tn;
  // Tiles are numbered in groups of GROUP tile rows, column by column inside a group, so the workgroups
  // an XCD runs side by side form a GROUP x 8 patch that shares GROUP left and 8 right operand tiles.
  constexpr int GROUP = 4;
  if (P.tile_mode == 2) {
    // only the tiles with tn >= tm exist: a group holds a small triangle, then full columns
    const int T = P.tiles_n;
    int first = 0, gs, tri;
    for (;;) {
      gs = min(GROUP, T - first);
      tri = gs * (gs + 1) / 2;
      const int cnt = tri + gs * (T - first - gs);
      if (id < cnt) break;
      id -= cnt;
      first += gs;
    }
    if (id < tri) {
      int c = 0;
      while (id > c) { id -= c + 1; ++c; }
      tm = first + id;
      tn = first + c;
    } else {
      id -= tri;
      tn = first + gs + id / gs;
      tm = first + id % gs;
    }
  } else {
    const int width = GROUP * P.tiles_n;
    const int g = id / width, first = g * GROUP;
    const int gsz = min(P.tiles_m - first, GROUP);
    const int r = id - g * width;
    tm = first + r % gsz;
    tn = r / gsz;
  }
  const int m0 = tm * BT, n0 = tn * BT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int rl = lane & 31, half = lane >> 5;

  const bool skipped = P.tile_mode == 1 && n0 + BT <= m0;
  int klo = 0, khi = P.K;
  if (P.k_mode == 1) klo = min(n0, P.K);
  if (P.k_mode == 2) { klo = min(m0, P.K); khi = min(P.K, n0 + BT); }
  const int nk = (skipped || khi <= klo) ? 0 : (khi - klo) / kGemmBK;

  f32x16 acc[FR][FR];
#pragma unroll
  for (int i = 0; i < FR; ++i)
#pragma unroll
    for (int j = 0; j < FR; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  if (P.nterm > 1) {
    if (P.kind == 0) tile_loop<BT, 0, true>(P, smem, m0, n0, klo, nk, acc);
    else if (P.kind == 1) tile_loop<BT, 1, true>(P, smem, m0, n0, klo, nk, acc);
    else tile_loop<BT, 2, true>(P, smem, m0, n0, klo, nk, acc);
  } else {
    if (P.kind == 0) tile_loop<BT, 0, false>(P, smem, m0, n0, klo, nk, acc);
    else if (P.kind == 1) tile_loop<BT, 1, false>(P, smem, m0, n0, klo, nk, acc);
    else tile_loop<BT, 2, false>(P, smem, m0, n0, klo, nk, acc);
  }

  // ---- epilogue.  MFMA 32x32 result: register v of a lane holds row 8*(v/4) + 4*(lane/32) + v%4,
  // column lane%32 of the block.
  // For C += acc all 64 loads of a row of blocks are issued before the first store, so the
  // read-modify-write costs a few memory round trips per tile instead of one per element.
  if (skipped && P.store_mode == 0) return;
  const int rbase = m0 + wm * WT + 4 * half, cbase = n0 + wn * WT + rl;
  if (P.store_mode == 0) {
#pragma unroll
    for (int i = 0; i < FR; ++i) {
      float old[FR][16];
#pragma unroll
      for (int j = 0; j < FR; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rbase + i * 32 + 8 * (v >> 2) + (v & 3), col = cbase + j * 32;
          old[j][v] = (row < P.M && col < P.N) ? P.C[(int64_t)row * P.ldc + col] : 0.f;
        }
#pragma unroll
      for (int j = 0; j < FR; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rbase + i * 32 + 8 * (v >> 2) + (v & 3), col = cbase + j * 32;
          if (row < P.M && col < P.N) P.C[(int64_t)row * P.ldc + col] = old[j][v] + acc[i][j][v];
        }
    }
  } else {
#pragma unroll
    for (int i = 0; i < FR; ++i)
#pragma unroll
      for (int j = 0; j < FR; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rbase + i * 32 + 8 * (v >> 2) + (v & 3), col = cbase + j * 32;
          if (row < P.M && col < P.N) {
            const float a = acc[i][j][v];
            P.C[(int64_t)row * P.ldc + col] = (P.store_mode == 1 || col > row) ? a : 0.f;
          }
        }
  }
}

// CAPPED = false: one workgroup per tile.  CAPPED = true: a workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x,
// ...: the caller caps the grid to leave compute units to a kernel running beside this one.  The grid is a multiple
// of 8 then, so a workgroup's tiles all belong to its own XCD's share.
template <int BT, bool CAPPED>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmBatch b) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  if (!CAPPED) {
    gemm_tile<BT>(b, smem, blockIdx.x);
  } else {
    const int total = b.ntiles[0] + b.ntiles[1];
    for (int wid = blockIdx.x; wid < total; wid += gridDim.x) {
      gemm_tile<BT>(b, smem, wid);
      __syncthreads();                   // the last fragment reads of this tile before the next tile's loads land in LDS
    }
  }
}

static LdsLimitOnce g_lds256, g_lds128, g_lds256c, g_lds128c;
hipError_t launch_gemm(const GemmBatch& b, hipStream_t s) {
  GemmBatch bb = b;
  int total = 0;
  for (int i = 0; i < 2; ++i) {
    const GemmProblem& q = bb.p[i];
    bb.ntiles[i] = i >= bb.nprob ? 0 : q.tile_mode == 2 ? q.tiles_m * (q.tiles_m + 1) / 2 : q.tiles_m * q.tiles_n;
    total += bb.ntiles[i];
  }
  if (total == 0) return hipSuccess;
  hipError_t e = g_lds256.ensure(reinterpret_cast<const void*>(&gemm_nt_kernel<256, false>), kLds256);
  if (e == hipSuccess) e = g_lds128.ensure(reinterpret_cast<const void*>(&gemm_nt_kernel<128, false>), kLds128);
  if (e == hipSuccess) e = g_lds256c.ensure(reinterpret_cast<const void*>(&gemm_nt_kernel<256, true>), kLds256);
  if (e == hipSuccess) e = g_lds128c.ensure(reinterpret_cast<const void*>(&gemm_nt_kernel<128, true>), kLds128);
  if (e != hipSuccess) return e;
  if (b.max_wgs > 0 && b.max_wgs < total) {
    const int grid = b.max_wgs >= 8 ? b.max_wgs / 8 * 8 : 8;
    if (b.tile == 256)
      hipLaunchKernelGGL((gemm_nt_kernel<256, true>), dim3(grid), dim3(256), kLds256, s, bb);
    else
      hipLaunchKernelGGL((gemm_nt_kernel<128, true>), dim3(grid), dim3(256), kLds128, s, bb);
  } else if (b.tile == 256) {
    hipLaunchKernelGGL((gemm_nt_kernel<256, false>), dim3(total), dim3(256), kLds256, s, bb);
  } else {
    hipLaunchKernelGGL((gemm_nt_kernel<128, false>), dim3(total), dim3(256), kLds128, s, bb);
  }
  return hipGetLastError();
}

}  // namespace gptaq
