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

namespace gptaq {

template <int BT>
__global__ __launch_bounds__(256) void gemm_nt_kernel(GemmBatch b) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int WT = BT / 2;             // wave tile edge
  constexpr int FR = WT / 32;            // 32x32 MFMA blocks per wave tile edge
  constexpr int NP = BT / 32;            // 32-row passes of the global->LDS copy
  constexpr int OPB = BT * 128;          // bytes of one operand k-tile

  // ---- which tile: spread consecutive tiles over one XCD so they share operands in its L2
  const int total = gridDim.x;
  int id = blockIdx.x;
  {
    const int per = total >> 3, rem = total & 7, xcd = id & 7, loc = id >> 3;
    id = xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
  }
  int pi = 0;
  {
    const int t0 = b.p[0].tiles_m * b.p[0].tiles_n;
    if (id >= t0) { pi = 1; id -= t0; }
  }
  const GemmProblem& P = b.p[pi];
  int tm, tn;
  {
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
    const uint16_t* lp = sg.L + (int64_t)(m0 + crow) * sg.ldl + k + cchunk * 8;
    const uint16_t* rp = sg.R + (int64_t)(n0 + crow) * sg.ldr + k + cchunk * 8;
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

  if (total_it > 0) {
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int it = 0; it < total_it; ++it) {
      const bool more = it + 1 < total_it;
      if (more) load_global(it + 1);
      const unsigned char* lb = smem + (it & 1) * 2 * OPB + (wm * WT + rl) * 128;
      const unsigned char* rb = smem + (it & 1) * 2 * OPB + OPB + (wn * WT + rl) * 128;
#pragma unroll
      for (int kk = 0; kk < kGemmBK / 16; ++kk) {
        const int off = ((kk * 2 + half) ^ sw) << 4;
        bf16x8 af[FR], bfr[FR];
#pragma unroll
        for (int i = 0; i < FR; ++i) {
          af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(lb + i * 32 * 128 + off));
          bfr[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(rb + i * 32 * 128 + off));
        }
#pragma unroll
        for (int i = 0; i < FR; ++i)
#pragma unroll
          for (int j = 0; j < FR; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
      if (more) store_lds((it + 1) & 1);
      __syncthreads();
    }
  }

  // ---- epilogue.  MFMA 32x32 result: register v of a lane holds row 8*(v/4) + 4*(lane/32) + v%4,
  // column lane%32 of the block.
  if (skipped && P.store_mode == 0) return;
#pragma unroll
  for (int i = 0; i < FR; ++i)
#pragma unroll
    for (int j = 0; j < FR; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * WT + i * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
        const int col = n0 + wn * WT + j * 32 + rl;
        if (row < P.M && col < P.N) {
          float* c = P.C + (int64_t)row * P.ldc + col;
          const float a = acc[i][j][v];
          if (P.store_mode == 0) *c += a;
          else if (P.store_mode == 1) *c = a;
          else *c = col > row ? a : 0.f;
        }
      }
}

static bool g_attr_set = false;

hipError_t launch_gemm(const GemmBatch& b, hipStream_t s) {
  int total = 0;
  for (int i = 0; i < b.nprob; ++i) total += b.p[i].tiles_m * b.p[i].tiles_n;
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
  GemmBatch bb = b;
  if (bb.nprob == 1) { bb.p[1].tiles_m = 0; bb.p[1].tiles_n = 0; }
  if (b.tile == 256)
    hipLaunchKernelGGL(gemm_nt_kernel<256>, dim3(total), dim3(256), 4 * 256 * 128, s, bb);
  else
    hipLaunchKernelGGL(gemm_nt_kernel<128>, dim3(total), dim3(256), 4 * 128 * 128, s, bb);
  return hipGetLastError();
}

}  // namespace gptaq
