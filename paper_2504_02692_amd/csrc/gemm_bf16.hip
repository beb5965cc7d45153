// bf16 x bf16 -> fp32 MFMA GEMM for gfx950:  C (+)= sum_s L_s R_s^T.
//
// Every dense contraction of the solve goes through this kernel (Algorithm 1 line 2: H and
// dXXT; line 4: the two products of Theorem 4.2; lines 11-12: the lazy trailing update of
// Eq. 18).  fp32-accurate products are obtained by splitting an fp32 operand into bf16
// terms and listing the cross products as K-segments.
//
// Tiling: a 256-thread workgroup owns a BT x BT tile of C (BT = 256 or 128); its four
// wavefronts sit 2 x 2 and each accumulates a (BT/2)^2 sub-tile with
// v_mfma_f32_32x32x16_bf16 (accumulators in AGPRs).  Operand k-tiles (BT rows x 32 bf16) go
// from global memory straight into LDS (global_load_lds_dwordx4, no VGPR staging) through a
// ring of four LDS stages, three k-tiles ahead of the multiply; fragment reads are
// ds_read_b128 on an XOR-swizzled layout and run one k-step ahead of the MFMAs.
#include "common.h"

namespace gptaq {

template <int BT>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmBatch b) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int WT = BT / 2;             // wave tile edge
  constexpr int FR = WT / 32;            // 32x32 MFMA blocks per wave tile edge
  constexpr int OPB = BT * 64;           // bytes of one operand k-tile (BT rows x 32 bf16)
  constexpr int STAGE_BYTES = 2 * OPB;
  constexpr int NSTAGE = 4;
  constexpr int LPW = BT / 64;           // 1 KB wave-loads per operand per wave per k-tile

  // ---- which tile.  Workgroups are dealt round-robin to the 8 XCDs; inside each problem, give every
  // XCD one contiguous run of tiles so that they share operand tiles in that XCD's L2, and so that
  // every XCD gets the same share of each problem (the problems differ in K).
  int id = blockIdx.x;
  int pi = 0;
  int ntile = b.ntiles[0];
  if (id >= ntile) { pi = 1; id -= ntile; ntile = b.ntiles[1]; }
  {
    const int per = ntile >> 3, rem = ntile & 7, xcd = id & 7, loc = id >> 3;
    id = xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
  }
  const GemmProblem& P = b.p[pi];
  int tm, tn;
  if (P.tile_mode == 2) {
    // only the tiles with tn >= tm exist, numbered row by row
    tm = 0;
    int rowlen = P.tiles_n;
    while (id >= rowlen) { id -= rowlen; --rowlen; ++tm; }
    tn = tm + id;
  } else {
    constexpr int GROUP = 4;
    const int width = GROUP * P.tiles_n;
    const int g = id / width, first = g * GROUP;
    const int gsz = min(P.tiles_m - first, GROUP);
    const int r = id - g * width;
    tm = first + r % gsz;
    tn = r / gsz;
  }
  const int m0 = tm * BT, n0 = tn * BT;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const bool skipped = P.tile_mode == 1 && n0 + BT <= m0;
  int klo = 0, khi = P.K;
  if (P.k_mode == 1) klo = min(n0, P.K);
  if (P.k_mode == 2) { klo = min(m0, P.K); khi = min(P.K, n0 + BT); }
  const int nk = (skipped || khi <= klo) ? 0 : (khi - klo) / kGemmBK;
  const int total_it = nk * P.nseg;

  f32x16 acc[FR][FR];
#pragma unroll
  for (int i = 0; i < FR; ++i)
#pragma unroll
    for (int j = 0; j < FR; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // ---- LDS tile format.  An operand k-tile is BT rows x 32 bf16 (64 B per row).  The LDS of gfx950
  // has 64 banks (256 B per clock), and a ds_read_b128 serves 16 lanes per clock, so 16 consecutive
  // fragment rows of one 16-byte chunk column must land in 16 different 16-byte slots of a 256-byte
  // line.  Four rows share a line; slot = (row & 3) * 4 + (chunk ^ (line & 3)): the four lines that
  // 16 consecutive rows touch use four different XOR values, i.e. disjoint slot sets.
  // Loads go global -> LDS directly (global_load_lds_dwordx4): lane l of a wave writes the 16 bytes at
  // LDS base + 16 l, so a wave fills 4 consecutive lines (16 rows) and each lane fetches the
  // (row, chunk) that belongs in its slot.
  const int ld_line = lane >> 4;                            // line inside the wave's 4 lines
  const int ld_row = ld_line * 4 + ((lane & 15) >> 2);      // row inside the wave's 16 rows
  const int ld_chunk = (lane & 3) ^ ld_line;                // undo the XOR (line & 3 == ld_line)
  auto issue_loads = [&](int it) {
    const int s = it / nk;
    const int64_t kt = (klo / kGemmBK) + (it - s * nk);
    const GemmSeg& sg = P.seg[s];
    const int stage = it % NSTAGE;
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
      const int r = (wave * LPW + j) * 16 + ld_row;
      const uint16_t* lp = sg.L + (int64_t)(m0 + r) * sg.ldl + kt * sg.ktl + ld_chunk * 8;
      const uint16_t* rp = sg.R + (int64_t)(n0 + r) * sg.ldr + kt * sg.ktr + ld_chunk * 8;
      unsigned char* dl = smem + stage * STAGE_BYTES + (wave * LPW + j) * 1024;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)lp,
                                       (__attribute__((address_space(3))) void*)dl, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)rp,
                                       (__attribute__((address_space(3))) void*)(dl + OPB), 16, 0, 0);
    }
  };

  // fragment reads: lane -> row (lane & 31) of a 32-row block, chunk 2 kk + (lane >> 5)
  const int rl = lane & 31, half = lane >> 5;
  const int fr_line = rl >> 2, fr_x = fr_line & 3, fr_hi = (rl & 3) << 2;
  bf16x8 af[2][FR], bfr[2][FR];
  auto read_frags = [&](int stage, int kk, int set) {
    const unsigned char* lb = smem + stage * STAGE_BYTES + (wm * (WT / 4) + fr_line) * 256;
    const unsigned char* rb = smem + stage * STAGE_BYTES + OPB + (wn * (WT / 4) + fr_line) * 256;
    const int off = (fr_hi | ((kk * 2 + half) ^ fr_x)) << 4;
#pragma unroll
    for (int i = 0; i < FR; ++i) {
      af[set][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(lb + i * 8 * 256 + off));
      bfr[set][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(rb + i * 8 * 256 + off));
    }
  };
  auto mfma_step = [&](int set) {
#pragma unroll
    for (int i = 0; i < FR; ++i)
#pragma unroll
      for (int j = 0; j < FR; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bfr[set][j], acc[i][j], 0, 0, 0);
  };
  // wait until at most `tiles` k-tiles of this wave's own loads are still in flight (loads return in
  // order), and all LDS reads have returned
  auto wait_tiles = [&](int tiles) {
    constexpr int T1 = 2 * LPW, T2 = 4 * LPW;
    if (tiles >= 2) __builtin_amdgcn_s_waitcnt(((T2 & 15) | ((T2 >> 4) << 14)) | (7 << 4));
    else if (tiles == 1) __builtin_amdgcn_s_waitcnt(((T1 & 15) | ((T1 >> 4) << 14)) | (7 << 4));
    else __builtin_amdgcn_s_waitcnt(7 << 4);
  };

  // Pipeline: k-tile `it` is multiplied from stage it % 4 while tiles it+1 .. it+3 are in flight or
  // landed.  One barrier per k-tile: it publishes tile it+1 (every wave waited for its own loads) and
  // retires stage (it - 1) % 4, which the loads issued at the top of the next iteration overwrite.
  if (total_it > 0) {
    for (int t = 0; t < NSTAGE - 1 && t < total_it; ++t) issue_loads(t);
    wait_tiles(min(total_it, NSTAGE - 1) - 1);
    __syncthreads();
    read_frags(0, 0, 0);
    for (int it = 0; it < total_it; ++it) {
      const int stage = it % NSTAGE;
      if (it + NSTAGE - 1 < total_it) issue_loads(it + NSTAGE - 1);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(stage, 1, 1);
      mfma_step(0);
      __builtin_amdgcn_sched_barrier(0);
      wait_tiles(min(total_it - 1, it + NSTAGE - 1) - (it + 1));
      __syncthreads();
      __builtin_amdgcn_sched_barrier(0);
      if (it + 1 < total_it) read_frags((it + 1) % NSTAGE, 0, 0);
      mfma_step(1);
      __builtin_amdgcn_sched_barrier(0);
    }
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

static bool g_attr_set = false;

hipError_t launch_gemm(const GemmBatch& b, hipStream_t s) {
  GemmBatch bb = b;
  int total = 0;
  for (int i = 0; i < 2; ++i) {
    const GemmProblem& q = bb.p[i];
    bb.ntiles[i] = i >= bb.nprob ? 0 : q.tile_mode == 2 ? q.tiles_m * (q.tiles_m + 1) / 2 : q.tiles_m * q.tiles_n;
    total += bb.ntiles[i];
  }
  if (total == 0) return hipSuccess;
  if (!g_attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<256>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 2 * 256 * 64);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<128>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 2 * 128 * 64);
    if (e != hipSuccess) return e;
    g_attr_set = true;
  }
  if (b.tile == 256)
    hipLaunchKernelGGL(gemm_nt_kernel<256>, dim3(total), dim3(256), 4 * 2 * 256 * 64, s, bb);
  else
    hipLaunchKernelGGL(gemm_nt_kernel<128>, dim3(total), dim3(256), 4 * 2 * 128 * 64, s, bb);
  return hipGetLastError();
}

}  // namespace gptaq
