// bf16 x bf16 -> fp32 MFMA GEMM for gfx950:  C (+)= sum_s L_s R_s^T.
//
// Every dense contraction of the solve goes through this kernel (Algorithm 1 line 2: H and
// dXXT; line 4: the two products of Theorem 4.2; lines 11-12: the lazy trailing update of
// Eq. 18).  fp32-accurate products are obtained by splitting an fp32 operand into bf16
// terms and listing the cross products as K-segments.
//
// Tiling: a 256-thread workgroup owns a BT x BT tile of C (BT = 256 or 128); its four
// wavefronts sit 2 x 2 and each accumulates a (BT/2)^2 sub-tile with
// v_mfma_f32_32x32x16_bf16.  Operand k-tiles (BT rows x 64 bf16) are staged through LDS in
// 16-byte chunks whose position inside a 128-byte row is XOR-ed with the row number, which
// makes both the global->LDS writes and the ds_read_b128 fragment reads bank-conflict free.
// Two LDS stages, one barrier per k-tile; the next k-tile is in flight in registers while
// the current one is multiplied.
#include "common.h"
#include <cstdlib>

namespace gptaq {

template <int BT, int DBG = 0>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmBatch b) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int WT = BT / 2;             // wave tile edge
  constexpr int FR = WT / 32;            // 32x32 MFMA blocks per wave tile edge
  constexpr int NP = BT / 32;            // 32-row passes of the global->LDS copy
  constexpr int OPB = BT * 128;          // bytes of one operand k-tile

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

  // global -> LDS copy roles
  const int crow = tid >> 3, cchunk = tid & 7;
  const int cst = crow * 128 + ((cchunk ^ (crow & 7)) << 4);
  // fragment read roles
  const int rl = lane & 31, half = lane >> 5, sw = lane & 7;

  u32x4 pl[NP], pr[NP];
  auto load_global = [&](int it) {
    const int s = it / nk;
    const int k = klo + (it - s * nk) * kGemmBK;
    const GemmSeg& sg = P.seg[s];
    const int64_t kt = k / kGemmBK;
    const uint16_t* lp = sg.L + (int64_t)(m0 + crow) * sg.ldl + kt * sg.ktl + cchunk * 8;
    const uint16_t* rp = sg.R + (int64_t)(n0 + crow) * sg.ldr + kt * sg.ktr + cchunk * 8;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      pl[p] = *reinterpret_cast<const u32x4*>(lp + (int64_t)p * 32 * sg.ldl);
      pr[p] = *reinterpret_cast<const u32x4*>(rp + (int64_t)p * 32 * sg.ldr);
    }
  };
  auto store_lds = [&](int buf) {
    unsigned char* lb = smem + buf * 2 * OPB;
    unsigned char* rb = lb + OPB;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
      *reinterpret_cast<u32x4*>(lb + cst + p * 32 * 128) = pl[p];
      *reinterpret_cast<u32x4*>(rb + cst + p * 32 * 128) = pr[p];
    }
  };

  // Fragment reads are software-pipelined by hand: while the 16 (or 4) MFMAs of k-step kk run, the
  // ds_read_b128 of k-step kk+1 are already in flight into the other register set; the LDS writes of
  // the next k-tile are issued under the MFMAs of the last k-step.  sched_barrier keeps the compiler
  // from re-serialising the phases.
  bf16x8 af[2][FR], bfr[2][FR];
  auto read_frags = [&](int buf, int kk, int set) {
    if ((DBG & 16) && !(buf == 0 && kk == 0)) return;
    const unsigned char* lb = smem + buf * 2 * OPB + (wm * WT + rl) * 128;
    const unsigned char* rb = smem + buf * 2 * OPB + OPB + (wn * WT + rl) * 128;
    const int off = ((kk * 2 + half) ^ sw) << 4;
#pragma unroll
    for (int i = 0; i < FR; ++i) {
      af[set][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(lb + i * 32 * 128 + off));
      bfr[set][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(rb + i * 32 * 128 + off));
    }
  };
  auto mfma_step = [&](int set) {
#pragma unroll
    for (int i = 0; i < FR; ++i)
#pragma unroll
      for (int j = 0; j < FR; ++j)
        if (!(DBG & 2) || (i == 0 && j == 0))
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[set][i], bfr[set][j], acc[i][j], 0, 0, 0);
  };

  if (total_it > 0) {
    load_global(0);
    store_lds(0);
    __syncthreads();
    read_frags(0, 0, 0);
    for (int it = 0; it < total_it; ++it) {
      const bool more = it + 1 < total_it;
      const int buf = it & 1;
      if (more && !(DBG & 1)) load_global(it + 1);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(buf, 1, 1);
      mfma_step(0);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(buf, 2, 0);
      mfma_step(1);
      __builtin_amdgcn_sched_barrier(0);
      read_frags(buf, 3, 1);
      mfma_step(0);
      __builtin_amdgcn_sched_barrier(0);
      if (more && !(DBG & 4)) store_lds(buf ^ 1);
      mfma_step(1);
      __builtin_amdgcn_sched_barrier(0);
      if (!(DBG & 8)) __syncthreads();
      if (more) read_frags(buf ^ 1, 0, 0);
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
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 256 * 128);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<128>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 128 * 128);
    if (e != hipSuccess) return e;
    g_attr_set = true;
  }
  static int dbg = getenv("GPTAQ_GEMM_DEBUG") ? atoi(getenv("GPTAQ_GEMM_DEBUG")) : 0;
  bb.debug = dbg;
  if (b.tile == 256 && dbg) {
    void (*k)(GemmBatch) = nullptr;
    switch (dbg) {
      case 5: k = gemm_nt_kernel<256, 5>; break;
      case 13: k = gemm_nt_kernel<256, 13>; break;
      case 29: k = gemm_nt_kernel<256, 29>; break;
      case 21: k = gemm_nt_kernel<256, 21>; break;
      case 4: k = gemm_nt_kernel<256, 4>; break;
      case 1: k = gemm_nt_kernel<256, 1>; break;
      default: return hipErrorInvalidValue;
    }
    hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 256 * 128);
    hipLaunchKernelGGL(k, dim3(total), dim3(256), 4 * 256 * 128, s, bb);
  } else if (b.tile == 256)
    hipLaunchKernelGGL(gemm_nt_kernel<256>, dim3(total), dim3(256), 4 * 256 * 128, s, bb);
  else
    hipLaunchKernelGGL(gemm_nt_kernel<128>, dim3(total), dim3(256), 4 * 128 * 128, s, bb);
  return hipGetLastError();
}

}  // namespace gptaq
