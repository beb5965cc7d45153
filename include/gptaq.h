/*
 * libgptaq - the GPTAQ per-layer asymmetric-calibration solve on one MI355X (gfx950).
 *
 * Three stages, in the order of Algorithm 1 of the paper (arXiv 2504.02692):
 *
 *   gptaq_accumulate      line 2   : H += X X^T,  dXXT += (X~ - X) X^T   (streamed over tokens)
 *   gptaq_prepare         lines 3-4: damping, H_lam^-1 = L L^T, U = L^T, and the fused
 *                                    correction matrix P = ((dXXT L) (.) M_U) L^T (Theorem 4.2)
 *   gptaq_quantize_layer  lines 5-13: the blocked column loop with lazy trailing updates
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates no
 *     device memory; scratch comes in through `ws` (size from the matching *_workspace_bytes).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it and the calls return without waiting for the GPU.
 *   - Matrices are row-major with a leading dimension in ELEMENTS.  Activations are
 *     token-major, (tokens x n): the transpose of the paper's n x k matrix X.
 *   - bf16 values travel as uint16_t bit patterns.
 *   - Return value: GPTAQ_OK or a negative GPTAQ_E* code for argument errors, detected on
 *     the host before anything is launched.  Numerical trouble (a non-positive pivot) is
 *     reported asynchronously through the caller's device `info` words.
 *   - Calls that share a workspace or an output must be ordered by the caller (same stream).
 */
#ifndef GPTAQ_H
#define GPTAQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GPTAQ_OK             0
#define GPTAQ_ENULL         -1   /* a required pointer is NULL                              */
#define GPTAQ_EDIM          -2   /* a dimension or leading dimension is out of range       */
#define GPTAQ_EUNSUPPORTED  -3   /* bits/group/blocksize combination not supported         */
#define GPTAQ_EWORKSPACE    -4   /* workspace too small or misaligned (needs 256 B)        */
#define GPTAQ_ELAUNCH       -5   /* the HIP runtime refused a launch; see gptaq_last_hip_error */
#define GPTAQ_ETOOLARGE     -6   /* beyond the fixed capacity of an entry point that allocates nothing */

/* Human-readable text for a status code. */
const char* gptaq_status_string(int status);
/* hipError_t of the most recent failed launch on this thread (0 if none). */
int gptaq_last_hip_error(void);

/* ---------------------------------------------------------------------------------------
 * Algorithm 1, line 2.  H += X^T X and dXXT += (X~ - X)^T X over `tokens` rows of the
 * token-major bf16 activations X (quantised model's input) and Xtilde (full-precision
 * model's input).  dXXT[q][j] = sum_t (X~[t][q] - X[t][q]) * X[t][j]  (row: neuron of dX,
 * column: neuron of X - the row vector dX_{q,:} X^T of Eq. 16).  Plain sums, fp32.
 *
 *   X, Xtilde : (tokens x n) bf16, leading dimension ldx >= n, ldx % 8 == 0, 16-byte aligned.
 *   H         : (n x n) fp32, ldh >= n.  Only the upper triangle (col >= row) is maintained;
 *               entries below the diagonal of H are never read and are left in an unspecified
 *               state (gptaq_symmetrize fills them).  Caller zero-initialises before the
 *               first chunk; call again with more tokens to continue the sums.
 *   dXXT      : (n x n) fp32, ldh >= n, all entries maintained (not symmetric).
 *   ws        : >= gptaq_accumulate_workspace_bytes(tokens, n) bytes, 256-byte aligned.  A
 *               smaller workspace is accepted down to the size for 64 tokens; the chunk is
 *               then processed in several passes.
 * dX is formed in fp32 and split exactly into two bf16 terms, so products are exact and
 * only fp32 accumulation rounding remains.
 */
size_t gptaq_accumulate_workspace_bytes(int64_t tokens, int64_t n);
int gptaq_accumulate(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                     int64_t ldx, float* H, float* dXXT, int64_t ldh,
                     void* ws, size_t ws_bytes, void* stream);

/* gptaq_accumulate for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same sums, same kernels; the
 * split operands go to a 32 MiB scratch array that is part of the library's code object (one copy per GPU,
 * held until the process ends), and the call makes no hipMalloc, hipFree or other allocating call.
 * The chunk is processed in passes of as many tokens as fit:
 * floor(32 MiB / (6 * round_up(n, tile))) rounded down to 64 (1344 tokens at n = 4096).
 *   n > 16384 returns GPTAQ_ETOOLARGE before anything is launched; other argument errors as gptaq_accumulate.
 *   Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two streams, two
 *   host threads) race.  Nothing in the array has to be cleared between calls. */
int gptaq_accumulate_noalloc(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                             int64_t ldx, float* H, float* dXXT, int64_t ldh, void* stream);

/* The same sums for callers that hand over small chunks, e.g. one 2048-token calibration sample at a time
 * (Section 5.1): a product launch has a fixed cost (its read-modify-write of H and dXXT, its last round of
 * tiles), so the chunk's operands are only appended to the workspace, and the products run once 32768
 * tokens are pending, or when `flush` is set.
 *   pending : HOST pointer, in/out: tokens staged in `ws` and not yet added to H and dXXT.  Start a series
 *             with 0 and keep passing the same workspace; H and dXXT are complete after a call with
 *             flush != 0 (which may bring tokens = 0), when *pending is 0 again.
 *   tokens  : a multiple of 64, except in the call with flush != 0.
 *   ws      : >= gptaq_accumulate_workspace_bytes(32768, n) bytes, 256-byte aligned; its contents belong
 *             to the series between calls.
 * Other arguments as for gptaq_accumulate.  A ragged chunk without flush, or *pending not a multiple of 64
 * in [0, 32768), is GPTAQ_EDIM. */
int gptaq_accumulate_staged(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                            int64_t ldx, float* H, float* dXXT, int64_t ldh,
                            void* ws, size_t ws_bytes, int64_t* pending, int flush, void* stream);

/* gptaq_accumulate and gptaq_accumulate_staged restricted to the part of dXXT that the solve reads when the
 * input channels are processed in their natural order.  Theorem 4.2 / Eq. 17 build P from dXXT L masked to its
 * STRICTLY UPPER triangle, with L lower triangular: entry (i, j) of the masked product is a sum over k >= j > i
 * of dXXT[i][k] L[k][j], so no entry of dXXT on or below its diagonal ever reaches P, U or a quantised weight.
 * These calls leave the products for that half out (two fifths of the matrix-core work of a launch):
 *   dXXT : on return the entries with col >= row hold the same sums, bit for bit, as after the full call; the
 *          entries below the diagonal are in an unspecified state (some tiles updated, others untouched).
 *          gptaq_prepare reads only the entries with col > row, so it returns the same U and P, bit for bit,
 *          as on the full matrix.
 *   NOT for act_order: gptaq_permute_hessian moves entries across the diagonal and needs the full matrix.
 * H and every other argument as for the full calls; a series may not mix full and upper calls if the lower
 * half is to mean anything. */
int gptaq_accumulate_upper(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                           int64_t ldx, float* H, float* dXXT, int64_t ldh,
                           void* ws, size_t ws_bytes, void* stream);
int gptaq_accumulate_staged_upper(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                                  int64_t ldx, float* H, float* dXXT, int64_t ldh,
                                  void* ws, size_t ws_bytes, int64_t* pending, int flush, void* stream);

/* Copies the upper triangle of the n x n fp32 matrix H onto its lower triangle. */
int gptaq_symmetrize(float* H, int64_t n, int64_t ldh, void* stream);

/* ---------------------------------------------------------------------------------------
 * Algorithm 1, lines 3-4.  Consumes H and dXXT.
 *   dead inputs (H_qq == 0): H_qq <- 1, row q of dXXT <- 0, dead[q] <- 1;
 *   lambda = damp * mean(diag H)  (damping relative to the mean diagonal, end of Section 4.2);
 *   H + lambda I = V V^T with V upper triangular, U = V^-1, so that (H + lambda I)^-1 = L L^T
 *   with L = U^T the lower factor of Step 3 / Lemma 4.1 (factorisation on fp64 data: its 64 x 64 blocks in
 *   fp64, its rank-256 block products in 46-bit row-scaled fixed point, exact in int32);
 *   P = ((dXXT L) (.) M_U) L^T = triu(dXXT U^T, 1) U   (Eq. 17).
 *
 *   H    : in: upper triangle of H.  out: U (upper triangular, zeros below), fp32.
 *   dXXT : in: dXXT; only the entries with col > row are read (Eq. 17 uses no others, see
 *          gptaq_accumulate_upper).  out: P (strictly upper triangular, zeros elsewhere).
 *   dead : n bytes, out: 1 for dead inputs else 0.  May be NULL.
 *   info : 2 x int32, out: info[0] = 0, or 1 + index of the first non-positive pivot, or -(1 + row) of a
 *          NaN/Inf entry found in H (upper triangle) or dXXT (strictly upper triangle) (in both cases U and P
 *          are garbage);
 *          info[1] = number of dead inputs.
 *   n    : at most 65280.
 * Streams: part of the factor sweep runs on a helper stream that the library creates once per device
 * (default priority, kept until the process ends) and ties to `stream` with events on both ends, so to
 * the caller the call is still one asynchronous operation on `stream`.  Host-side the call takes a
 * library lock: concurrent calls from several host threads are serialised while they enqueue.
 */
size_t gptaq_prepare_workspace_bytes(int64_t n);
int gptaq_prepare(float* H, float* dXXT, int64_t n, int64_t ldh, float damp,
                  uint8_t* dead, int32_t* info, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------
 * Algorithm 1, lines 5-13.  For every block of `blocksize` columns: quantise column by
 * column, all m rows in parallel, feeding  -E_j U[j, j:] + v_j P[j, j:]  to the remaining
 * columns of the block (E_j = (v_j - quant(v_j)) / U_jj, v_j the column's current value
 * just before it is quantised, Eq. 15), then apply the block's accumulated update to all
 * later columns at once (Eq. 18).  The result does not depend on blocksize.
 *
 *   W      : (m x n) fp32, ldw >= n.  in: weights.  out: dequantised quantised weights (Q).
 *   U, P   : outputs of gptaq_prepare, read-only, so one prepare serves every layer that
 *            shares the input (q/k/v, gate/up).
 *   dead   : n bytes from gptaq_prepare or NULL; dead columns of W are taken as 0.
 *   bits   : 2..8.  group: columns per (scale, zero) group, <= 0 for one group per row
 *            (range taken from the original row); else n % group == 0, blocksize % group == 0
 *            and group <= 128.  Group ranges come from the current (error-compensated)
 *            weights at the group's first column.  sym != 0: symmetric grid, zero = 2^(bits-1).
 *   blocksize : 1..128.
 *   codes  : (m x n) uint8, one code per byte, leading dimension n.
 *   scales, zeros : (m x G) fp32, G = max(1, n / group); zeros hold integers.
 *   ws     : >= gptaq_quantize_workspace_bytes(m, n) bytes, 256-byte aligned: the update operands (-E and V of a
 *            1024-column super-block for all rows, twice; the rows of U and P of EVERY super-block on the columns
 *            after it, as bf16 hi + lo: about 4 n^2 bytes, 0.46 GB at n = 11008, 11 GB at n = 53248).
 * Quantiser: range [min(0,min w), max(0,max w)], scale = (max-min)/(2^bits-1),
 * zero = rint(-min/scale), q = clamp(rint(w/scale)+zero), rint = half-to-even.
 */
size_t gptaq_quantize_workspace_bytes(int64_t m, int64_t n);
int gptaq_quantize_layer(float* W, int64_t m, int64_t n, int64_t ldw,
                         const float* U, const float* P, int64_t ldh, const uint8_t* dead,
                         int bits, int group, int sym, int blocksize,
                         uint8_t* codes, float* scales, float* zeros,
                         void* ws, size_t ws_bytes, void* stream);

/* The same solve with only some of the two update terms of Eq. 15 applied (the ablation of
 * Section 5.5): terms bit 0 = the quantisation-error term -E_j U[j, j:], bit 1 = the residual term
 * v_j P[j, j:].  3 = GPTAQ (gptaq_quantize_layer), 1 = GPTQ (P may be NULL), 2 = the second term
 * alone, 0 = round to nearest.  All other arguments as in gptaq_quantize_layer. */
int gptaq_quantize_layer_terms(float* W, int64_t m, int64_t n, int64_t ldw,
                               const float* U, const float* P, int64_t ldh, const uint8_t* dead,
                               int bits, int group, int sym, int blocksize,
                               uint8_t* codes, float* scales, float* zeros,
                               void* ws, size_t ws_bytes, void* stream, int terms);

/* The same solve with the clip-range search of Section 5.1 for the weight grid (the range that
 * minimises the squared quantisation error): whenever a (scale, zero) pair is taken from a range, the candidates
 * p = 1 - i / mse_grid, i = 0 .. mse_steps - 1, shrink that range about its zero-point
 * (scale_i = p * scale_0, same zero-point); the candidate with the smallest sum of squared
 * quantisation errors over the row-group is used (the earlier one on ties).  mse_steps = 0 is the
 * plain min-max grid; GPTQ's customary setting is mse_grid = 100, mse_steps = 80.
 * terms as in gptaq_quantize_layer_terms (3 = both). */
int gptaq_quantize_layer_ex(float* W, int64_t m, int64_t n, int64_t ldw,
                            const float* U, const float* P, int64_t ldh, const uint8_t* dead,
                            int bits, int group, int sym, int blocksize,
                            uint8_t* codes, float* scales, float* zeros,
                            void* ws, size_t ws_bytes, void* stream,
                            int terms, int mse_grid, int mse_steps);

/* ---------------------------------------------------------------------------------------
 * act_order (Sections 5.2, 5.3): quantise the input channels in the order of decreasing Hessian
 * diagonal.  The solve is unchanged; these calls permute its inputs and scatter its outputs back:
 *
 *   gptaq_act_order(H) -> perm;  gptaq_permute_hessian(H, dXXT, perm);  Wp = W[:, perm];
 *   gptaq_prepare;  gptaq_quantize_layer(Wp ...);  W^[:, perm] = Wp^;  codes[:, perm] = codes_p.
 *
 * Groups are groups of consecutive PERMUTED columns: original column perm[i] belongs to group
 * i / group, and scales / zeros are indexed by that group.
 *
 * gptaq_act_order: perm[r] = index of the input with the r-th largest H[i][i]; equal diagonals keep
 *   their index order.  perm: n x int32 (device).  ldh == 0: H points at the n diagonal entries themselves.
 * gptaq_permute_hessian: in place H[i][j] <- H[perm[i]][perm[j]] (upper triangle in; the whole symmetric
 *   matrix out) and dXXT[i][j] <- dXXT[perm[i]][perm[j]];  ws: gptaq_permute_hessian_workspace_bytes(n).
 * gptaq_permute_columns_{f32,u8}: inverse == 0: out[r][i] = in[r][perm[i]];
 *   inverse != 0: out[r][perm[i]] = in[r][i].  in and out must not overlap.
 */
int gptaq_act_order(const float* H, int64_t n, int64_t ldh, int32_t* perm, void* stream);

/* act_order with the upper-triangle accumulation (gptaq_accumulate_upper): the order has to be known BEFORE the sums
 * are taken, because which of dXXT[a][b] and dXXT[b][a] Eq. 17 reads depends on which of a and b comes first.  Two
 * passes over the layer's calibration inputs:
 *   pass 1: gptaq_accumulate_diag for every chunk (diag[j] += sum_t X[t][j]^2, the diagonal of H; diag: n x fp32,
 *           zero-initialised by the caller); gptaq_act_order(diag, n, 0, perm); gptaq_invert_permutation(perm, n, inv)
 *           (inv[perm[r]] = r; perm must be a permutation of 0 .. n-1);
 *   pass 2: gptaq_accumulate_upper_permuted for every chunk: gptaq_accumulate_upper on the inputs with their channels
 *           reordered, H[i][j] = sum_t X[t][perm[i]] X[t][perm[j]], dXXT likewise: what gptaq_permute_hessian makes
 *           of the full sums, on and above the diagonal, bit for bit, with no n x n permutation pass and two fifths
 *           less matrix-core work.  Then gptaq_prepare, Wp = W[:, perm], gptaq_quantize_layer as above.
 * The diagonal of pass 1 is summed in another order than the one inside H, so two inputs whose diagonals agree to
 * fp32 rounding may swap places against gptaq_act_order(H); any order is a valid one for the solve.
 * Other arguments as for gptaq_accumulate_upper.  inv_perm: n x int32 (device). */
int gptaq_accumulate_diag(const uint16_t* X, int64_t tokens, int64_t n, int64_t ldx, float* diag, void* stream);
int gptaq_invert_permutation(const int32_t* perm, int64_t n, int32_t* inv, void* stream);
int gptaq_accumulate_upper_permuted(const uint16_t* X, const uint16_t* Xtilde, int64_t tokens, int64_t n,
                                    int64_t ldx, const int32_t* inv_perm, float* H, float* dXXT, int64_t ldh,
                                    void* ws, size_t ws_bytes, void* stream);
size_t gptaq_permute_hessian_workspace_bytes(int64_t n);
int gptaq_permute_hessian(float* H, float* dXXT, int64_t n, int64_t ldh, const int32_t* perm,
                          void* ws, size_t ws_bytes, void* stream);
int gptaq_permute_columns_f32(const float* in, float* out, int64_t m, int64_t n, int64_t ldin,
                              int64_t ldout, const int32_t* perm, int inverse, void* stream);
int gptaq_permute_columns_u8(const uint8_t* in, uint8_t* out, int64_t m, int64_t n, int64_t ldin,
                             int64_t ldout, const int32_t* perm, int inverse, void* stream);

/* ---------------------------------------------------------------------------------------
 * Neighbours of the solve in the whole-model procedure (Algorithm 2).
 *
 * gptaq_fake_quant_activations: the activation quantiser of Section 5.1 (per token, asymmetric,
 *   clipping ratio `clip`, 0.9 in the paper), used to produce X when activations are quantised before
 *   the weights.  For every token row: range = clip * [min(0, min x), max(0, max x)],
 *   scale = fp32(range / (2^bits - 1)), zero = rint(-clip*min/scale),
 *   y = bf16(scale * (clamp(rint(x / scale) + zero) - zero)): rint(x / scale) is the exact rounding for the fp32 scale,
 *   the product is exact, one rounding to bf16.
 *   X, Y: (tokens x n) bf16, leading dimensions ldx, ldy; Y may equal X.
 * gptaq_pack_codes: packed row r = little-endian bit stream of the row's codes, code j in bits
 *   [j*bits, (j+1)*bits); gptaq_packed_words_per_row(n, bits) = ceil(n*bits/32) uint32 words per row.
 */
int gptaq_fake_quant_activations(const uint16_t* X, uint16_t* Y, int64_t tokens, int64_t n,
                                 int64_t ldx, int64_t ldy, int bits, float clip, void* stream);
int64_t gptaq_packed_words_per_row(int64_t n, int bits);
int gptaq_pack_codes(const uint8_t* codes, int64_t m, int64_t n, int64_t ldc, int bits,
                     uint32_t* packed, void* stream);

/* ---------------------------------------------------------------------------------------
 * Measurement aid (not part of the method).  While enabled, the library brackets its kernels
 * with HIP events on the caller's stream, grouped by tag:
 *   0 accumulate MFMA GEMM (H and dXXT, one launch per pass)   1 accumulate split/transpose pass
 *   2 factorisation + triangular inverse sweep (whole sweep)    3 the two Theorem-4.2 GEMMs
 *   4 column-loop kernel (one per block)                        5 trailing-update GEMM (one per block)
 *   6 trailing operand split/transpose
 * gptaq_profile_enable(mask) clears the records and records the tags whose bit (1 << tag) is set
 * in `mask`; 0 stops recording.
 * gptaq_profile_read waits for the recorded events and returns the number of bracketed
 * launches of `tag` and their summed duration in milliseconds.  Not thread-safe.
 */
int gptaq_profile_enable(int mask);
int gptaq_profile_read(int tag, int64_t* launches, double* total_ms);

/* Measurement aid: the rate the bf16 matrix cores of this GPU sustain when they do nothing else - a loop of
 * independent 32x32x16 bf16 MFMAs on every compute unit, operands in registers - for about `millis`
 * milliseconds (1..2000), after one untimed launch of the same length.  The chip is power-limited, so the
 * rate depends on the operand data: random_data = 0 multiplies all-ones (the least switching activity),
 * 1 multiplies random signs and mantissas (the fair ceiling for a product of real data).
 *   ws     : >= 1 MiB of device memory, 256-byte aligned (scratch).
 *   tflops, clock_ghz : HOST pointers, out: the measured rate and the core clock during the loop.
 * Synchronous: returns after the measurement. */
int gptaq_measure_mfma_peak(int random_data, int millis, void* ws, size_t ws_bytes, double* tflops,
                            double* clock_ghz, void* stream);

/* Measurement aid: what a plain streaming copy reaches on this GPU, the practical HBM ceiling quoted beside the
 * nominal 8 TB/s.  Copies `bytes` (a multiple of 16, >= 4096) from the first half of `ws` to the second, `reps`
 * times after one untimed pass; *gbps = bytes read + bytes written per second, in GB/s (HOST pointer).
 *   ws : >= 2 * bytes of device memory, 256-byte aligned (contents are scratch).
 * Synchronous: returns after the measurement. */
int gptaq_measure_hbm_copy(size_t bytes, int reps, void* ws, size_t ws_bytes, double* gbps, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GPTAQ_H */
