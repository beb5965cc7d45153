// Internal declarations shared by the translation units of libgptaq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/gptaq.h"

namespace gptaq {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kGemmBK = 32;          // bf16 elements per k-tile of the MFMA GEMM

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// One term of a GEMM: up to two left and two right bf16 operands (hi, lo) sharing one layout.
// Element (row, k) of an operand sits at base + row * ld + (k / 32) * kt + k % 32:  ld = K, kt = 32
// for a plain row-major K-contiguous matrix;  ld = 32, kt = rows * 32 for the k-tile-major layout, in
// which the 32-wide k-tile of a block of rows is one contiguous run (no power-of-two row stride, so a
// tile's lines spread over all memory channels).
struct GemmTerm {
  const uint16_t* L[2];
  const uint16_t* R[2];
  int64_t ldl, ldr;
  int64_t ktl, ktr;
};

// C (+)= sum_t sum_pairs L R^T.  kind 0: L0 R0.  kind 1: L0 R0 + L1 R0 (two left operands share the
// right one).  kind 2: L0 R0 + L0 R1 + L1 R0 (hi/lo split of both sides, lo*lo dropped).
// Operand buffers are zero-padded to whole tiles in rows and to a multiple of kGemmBK in K, so the
// main loop needs no bounds checks; stores are bounded by M and N.
struct GemmProblem {
  float* C;
  int64_t ldc;
  int32_t M, N, K;       // K per term (multiple of kGemmBK)
  int32_t tiles_m, tiles_n;
  int32_t kind, nterm;
  int32_t tile_mode;     // 0: all tiles; 1: tiles entirely below the diagonal do no work (but store);
                         // 2: square problem, only tiles with tile column >= tile row are scheduled
  int32_t k_mode;        // 0: all k; 1: k >= first column of the tile; 2: tile row0 <= k < tile col end
  int32_t store_mode;    // 0: C += acc; 1: C = acc; 2: C = acc where col > row, else 0
  GemmTerm term[2];
};

struct GemmBatch {
  int32_t nprob;
  int32_t tile;          // 128 or 256 (square block tile)
  int32_t ntiles[2];     // filled by launch_gemm
  GemmProblem p[2];
};

// Enqueue the batch; problems are scheduled in order (put the heavier one first).
hipError_t launch_gemm(const GemmBatch& b, hipStream_t s);
// Row padding the GEMM expects from an operand with `rows` logical rows.
inline int gemm_tile_for(int64_t M, int64_t N) {
  // 256 x 256 tiles move the fewest bytes per flop but one workgroup fills a CU; use them only when they
  // still give every CU a tile, otherwise 128 x 128 tiles (two workgroups per CU).
  const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
  return (M >= 1024 && N >= 1024 && t256 >= 224) ? 256 : 128;
}

void set_last_hip_error(hipError_t e);

// Optional per-kernel timing with HIP events (gptaq_profile_* in the public header).
enum ProfTag { kProfAccumGemm = 0, kProfAccumSplit = 1, kProfFactor = 2, kProfPGemm = 3, kProfColumnLoop = 4,
               kProfTrailGemm = 5, kProfTrailSplit = 6, kProfTags = 7 };
bool prof_enabled(int tag);
void prof_mark(int tag, hipStream_t s, bool begin);
struct ProfScope {
  int tag; hipStream_t s; bool on;
  ProfScope(int t, hipStream_t st) : tag(t), s(st), on(prof_enabled(t)) { if (on) prof_mark(tag, s, true); }
  ~ProfScope() { if (on) prof_mark(tag, s, false); }
};

#define GPTAQ_LAUNCH_CHECK()                                   \
  do {                                                         \
    hipError_t e__ = hipGetLastError();                        \
    if (e__ != hipSuccess) { set_last_hip_error(e__); return GPTAQ_ELAUNCH; } \
  } while (0)

}  // namespace gptaq
