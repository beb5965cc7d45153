// Internal declarations shared by the translation units of libgptaq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <mutex>
#include <vector>
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
  int32_t deal;          // how the tile list is shared out to the 8 XCDs: 0: one contiguous run each (tiles of equal
                         // length); 1: dealt four tiles at a time (tile lengths that vary along the list: k_mode 1, 2)
  GemmTerm term[2];
};

struct GemmBatch {
  int32_t nprob;
  int32_t tile;          // 128 or 256 (square block tile)
  int32_t ntiles[2];     // filled by launch_gemm
  int32_t max_wgs;       // 0: one workgroup per tile; else at most this many workgroups, each taking several tiles
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

// fp64-grade rank-k products through digit-sliced int8 MFMA (gemm_i8s.hip).  A sliced operand holds
// kI8Planes digit planes of rows_pad x kI8MaxK signed bytes (rows_pad a multiple of 128; rows and k beyond the
// source are zero) and one power-of-two scale (its exponent) per row.
constexpr int kI8Planes = 6;
constexpr int kI8MaxK = 256;
struct I8Operand {
  uint8_t* planes;
  int32_t* scale;
  int64_t rows_pad;
  int64_t chunk_stride() const { return rows_pad * 32; }
  int64_t plane_stride() const { return rows_pad * kI8MaxK; }
  static size_t plane_bytes(int64_t rows_pad) { return (size_t)kI8Planes * rows_pad * kI8MaxK; }
};
struct I8Gemm {
  const uint8_t* A; int64_t a_plane, a_chunk; const int32_t* sa;
  const uint8_t* B; int64_t b_plane, b_chunk; const int32_t* sb;
  double* C; int64_t ldc;
  int32_t M, N, nchunk, beta, upper_only, tiles_m, tiles_n, ntile;
  double alpha;
};
// Slices the R x K matrix with element (r, k) at src[r * sr + k * sk] (one stride must be 1, K <= kI8MaxK).
hipError_t launch_slice_i8(const double* src, int64_t sr, int64_t sk, int R, int K, const I8Operand& o, hipStream_t s);
// C = beta C + alpha A B^T over rows [a_row0, a_row0 + M) of A and [b_row0, b_row0 + N) of B (offsets multiples
// of 128 and 64); upper_only skips the tiles entirely below the diagonal of C.
hipError_t launch_gemm_i8s(const I8Operand& A, int a_row0, const I8Operand& B, int b_row0, double* C, int64_t ldc, int M,
                           int N, int K, double alpha, int beta, int upper_only, hipStream_t s);

// Column loop + in-super-block updates of a whole super-block in one launch (quantize_sb.hip).
constexpr int kSbCols = 1024;       // columns per super-block
struct SbArgs {
  float* W; int64_t ldw; int m, n;
  int sb0, sbw;                      // first column and width (<= kSbCols) of the super-block
  const float* U; const float* P; int64_t ldh;
  const uint16_t* Nop[4];            // launch_near_operands output: U hi, U lo, P hi, P lo
  const uint8_t* dead;
  float maxq; int group, sym, G, terms;
  float* scales; float* zeros; uint8_t* codes;
  uint16_t *Eh, *El, *Vh, *Vl;       // -E and V of the super-block as bf16 hi/lo, row stride ldev (NULL: not wanted)
  int64_t ldev;
  int fast_rows;                     // rows of W and of codes may be stored 16 bytes at a time
};
// N4: four buffers of (kSbCols / 16) * kSbCols * 16 bf16 each.
hipError_t launch_near_operands(const float* U, const float* P, int64_t ldh, int n, int sb0, int sbw, uint16_t* const* N4,
                                hipStream_t s);
hipError_t launch_quant_sb(const SbArgs& a, hipStream_t s);

void set_last_hip_error(hipError_t e);

// Helper stream of the library: entry points that run two chains of kernels side by side (the factor sweep of
// gptaq_prepare, the far updates of gptaq_quantize_layer) put one chain on the caller's stream and the other on this
// stream, tied together with events on both ends, so that to the caller the call is still one asynchronous
// operation on its own stream.  One stream (default priority) and one growing pool of events per device, created on
// first use and kept until the process ends.  The mutex serialises the host threads that enqueue through it.
struct SideStream {
  hipStream_t stream = nullptr;
  std::vector<hipEvent_t> events;
};
std::mutex& side_stream_mutex();
// The current device's helper stream with at least `nevents` events; nullptr on failure (call with the mutex held).
SideStream* side_stream(int nevents);

// Raises a kernel's dynamic LDS limit exactly once per process, whichever host thread comes first; every caller
// gets the result of that one attempt.
struct LdsLimitOnce {
  std::once_flag once;
  hipError_t result = hipSuccess;
  hipError_t ensure(const void* kernel, int bytes) {
    std::call_once(once, [&] { result = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
    return result;
  }
};

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
