// Host-side check of the argument-validation paths of libgptaq under AddressSanitizer and
// UndefinedBehaviorSanitizer (host code only; no GPU is needed: every call below must return its error code
// before anything is launched).  Built and run by tests/host_sanitizer_check.py.
#include "gptaq.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>

static int failures = 0;
#define EXPECT(call, want)                                                                   \
  do {                                                                                       \
    const int got_ = (call);                                                                 \
    if (got_ != (want)) { std::printf("FAIL %s: %d, expected %d\n", #call, got_, (want)); ++failures; } \
  } while (0)

int main() {
  // fake, suitably aligned non-null pointers: the entry points must not touch them before validating
  alignas(256) static unsigned char blob[4096];
  float* f = reinterpret_cast<float*>(blob);
  uint16_t* h = reinterpret_cast<uint16_t*>(blob);
  uint8_t* b = blob;
  int32_t* i32 = reinterpret_cast<int32_t*>(blob);
  uint32_t* u32 = reinterpret_cast<uint32_t*>(blob);
  void* ws = blob;
  int64_t pending = 0;

  for (int s = 0; s >= -7; --s)
    if (!gptaq_status_string(s) || !std::strlen(gptaq_status_string(s))) { std::printf("FAIL status string %d\n", s); ++failures; }

  // sizes: zero for non-positive arguments, monotone, no overflow trap at the largest supported n
  if (gptaq_accumulate_workspace_bytes(0, 16) != 0 || gptaq_accumulate_workspace_bytes(16, 0) != 0) { std::printf("FAIL accumulate ws 0\n"); ++failures; }
  if (gptaq_prepare_workspace_bytes(0) != 0 || gptaq_prepare_workspace_bytes(-5) != 0) { std::printf("FAIL prepare ws 0\n"); ++failures; }
  if (gptaq_quantize_workspace_bytes(0, 8) != 0 || gptaq_quantize_workspace_bytes(8, -1) != 0) { std::printf("FAIL quantize ws 0\n"); ++failures; }
  if (gptaq_prepare_workspace_bytes(65280) <= gptaq_prepare_workspace_bytes(53248)) { std::printf("FAIL prepare ws monotone\n"); ++failures; }
  if (gptaq_accumulate_workspace_bytes(32768, 65280) == 0 || gptaq_quantize_workspace_bytes(1 << 20, 65280) == 0) { std::printf("FAIL large ws\n"); ++failures; }
  (void)gptaq_permute_hessian_workspace_bytes(65280);
  if (gptaq_packed_words_per_row(4096, 4) != 512 || gptaq_packed_words_per_row(100, 3) != 10) { std::printf("FAIL packed words\n"); ++failures; }

  // accumulate
  EXPECT(gptaq_accumulate(nullptr, h, 64, 64, 64, f, f, 64, ws, 1 << 20, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate(h, h, 64, 64, 64, nullptr, f, 64, ws, 1 << 20, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate(h, h, 64, 64, 64, f, f, 64, nullptr, 1 << 20, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate(h, h, -1, 64, 64, f, f, 64, ws, 1 << 20, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate(h, h, 64, 0, 64, f, f, 64, ws, 1 << 20, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate(h, h, 64, 64, 32, f, f, 64, ws, 1 << 20, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate(h, h, 64, 64, 64, f, f, 8, ws, 1 << 20, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate(h, h, 64, 64, 64, f, f, 64, ws, 16, nullptr), GPTAQ_EWORKSPACE);
  EXPECT(gptaq_accumulate(h, h, 64, 64, 64, f, f, 64, blob + 8, 1 << 20, nullptr), GPTAQ_EWORKSPACE);
  EXPECT(gptaq_accumulate_noalloc(h, h, 64, 20000, 20000, f, f, 20000, nullptr), GPTAQ_ETOOLARGE);
  EXPECT(gptaq_accumulate_noalloc(nullptr, h, 64, 64, 64, f, f, 64, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate_noalloc(h, h, 64, 64, 8, f, f, 64, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate_staged(h, h, 64, 64, 64, f, f, 64, ws, 1 << 20, nullptr, 0, nullptr), GPTAQ_ENULL);
  pending = 40000;
  EXPECT(gptaq_accumulate_staged(h, h, 64, 64, 64, f, f, 64, ws, 1 << 20, &pending, 0, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate_upper(nullptr, h, 64, 64, 64, f, f, 64, ws, 1 << 20, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate_upper(h, h, 64, 60, 64, f, f, 64, ws, 1 << 20, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate_upper(h, h, 64, 64, 64, f, f, 64, ws, 16, nullptr), GPTAQ_EWORKSPACE);
  EXPECT(gptaq_accumulate_staged_upper(h, h, 64, 64, 64, f, f, 64, ws, 1 << 20, nullptr, 0, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate_staged_upper(h, h, 64, 64, 64, f, f, 64, ws, 1 << 20, &pending, 0, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate_upper_permuted(h, h, 64, 64, 64, nullptr, f, f, 64, ws, 1 << 20, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate_upper_permuted(h, h, 64, 64, 64, i32, f, f, 8, ws, 1 << 20, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_accumulate_diag(nullptr, 64, 64, 64, f, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_accumulate_diag(h, 64, 60, 64, f, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_invert_permutation(nullptr, 64, i32, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_invert_permutation(i32, -1, i32, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_symmetrize(nullptr, 64, 64, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_symmetrize(f, 64, 8, nullptr), GPTAQ_EDIM);

  // prepare
  EXPECT(gptaq_prepare(nullptr, f, 64, 64, 0.01f, nullptr, i32, ws, 1 << 30, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_prepare(f, f, 64, 64, 0.01f, nullptr, nullptr, ws, 1 << 30, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_prepare(f, f, 0, 64, 0.01f, nullptr, i32, ws, 1 << 30, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_prepare(f, f, 64, 8, 0.01f, nullptr, i32, ws, 1 << 30, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_prepare(f, f, 70000, 70000, 0.01f, nullptr, i32, ws, 1 << 30, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_prepare(f, f, 64, 64, -1.f, nullptr, i32, ws, 1 << 30, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_prepare(f, f, 64, 64, 0.01f, nullptr, i32, ws, 16, nullptr), GPTAQ_EWORKSPACE);
  EXPECT(gptaq_prepare(f, f, 64, 64, 0.01f, nullptr, i32, blob + 4, 1 << 30, nullptr), GPTAQ_EWORKSPACE);

  // quantize
  EXPECT(gptaq_quantize_layer(nullptr, 8, 64, 64, f, f, 64, nullptr, 4, 0, 0, 128, b, f, f, ws, 1 << 30, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_quantize_layer(f, 8, 64, 64, f, f, 64, nullptr, 4, 0, 0, 128, nullptr, f, f, ws, 1 << 30, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_quantize_layer(f, 0, 64, 64, f, f, 64, nullptr, 4, 0, 0, 128, b, f, f, ws, 1 << 30, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_quantize_layer(f, 8, 64, 8, f, f, 64, nullptr, 4, 0, 0, 128, b, f, f, ws, 1 << 30, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_quantize_layer(f, 8, 64, 64, f, f, 64, nullptr, 9, 0, 0, 128, b, f, f, ws, 1 << 30, nullptr), GPTAQ_EUNSUPPORTED);
  EXPECT(gptaq_quantize_layer(f, 8, 64, 64, f, f, 64, nullptr, 4, 48, 0, 128, b, f, f, ws, 1 << 30, nullptr), GPTAQ_EUNSUPPORTED);
  EXPECT(gptaq_quantize_layer(f, 8, 64, 64, f, f, 64, nullptr, 4, 0, 0, 1000, b, f, f, ws, 1 << 30, nullptr), GPTAQ_EUNSUPPORTED);
  EXPECT(gptaq_quantize_layer(f, 8, 64, 64, f, f, 64, nullptr, 4, 32, 0, 48, b, f, f, ws, 1 << 30, nullptr), GPTAQ_EUNSUPPORTED);
  EXPECT(gptaq_quantize_layer(f, 8, 64, 64, f, f, 64, nullptr, 4, 0, 0, 128, b, f, f, ws, 16, nullptr), GPTAQ_EWORKSPACE);
  EXPECT(gptaq_quantize_layer_terms(f, 8, 64, 64, f, f, 64, nullptr, 4, 0, 0, 128, b, f, f, ws, 1 << 30, nullptr, 7), GPTAQ_EUNSUPPORTED);
  EXPECT(gptaq_quantize_layer_ex(f, 8, 64, 64, f, f, 64, nullptr, 4, 0, 0, 128, b, f, f, ws, 1 << 30, nullptr, 3, 0, 5), GPTAQ_EUNSUPPORTED);

  // beside the main path
  EXPECT(gptaq_act_order(nullptr, 64, 64, i32, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_act_order(f, 64, 8, i32, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_permute_hessian(f, f, 64, 64, nullptr, ws, 1 << 30, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_permute_hessian(f, f, 64, 64, i32, ws, 16, nullptr), GPTAQ_EWORKSPACE);
  EXPECT(gptaq_permute_columns_f32(f, nullptr, 8, 64, 64, 64, i32, 0, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_permute_columns_f32(f, f + 512, 8, 64, 8, 64, i32, 0, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_permute_columns_u8(b, nullptr, 8, 64, 64, 64, i32, 0, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_fake_quant_activations(nullptr, h, 8, 64, 64, 64, 4, 0.9f, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_fake_quant_activations(h, h, 8, 64, 8, 64, 4, 0.9f, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_fake_quant_activations(h, h, 8, 64, 64, 64, 1, 0.9f, nullptr), GPTAQ_EUNSUPPORTED);
  EXPECT(gptaq_pack_codes(nullptr, 8, 64, 64, 4, u32, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_pack_codes(b, 8, 64, 64, 9, u32, nullptr), GPTAQ_EUNSUPPORTED);
  EXPECT(gptaq_profile_read(99, &pending, nullptr), GPTAQ_EDIM);
  EXPECT(gptaq_measure_mfma_peak(0, 10, nullptr, 0, nullptr, nullptr, nullptr), GPTAQ_ENULL);
  EXPECT(gptaq_measure_hbm_copy(1 << 20, 1, nullptr, 0, nullptr, nullptr), GPTAQ_ENULL);

  std::printf("%s: %d failure(s)\n", failures ? "FAILED" : "ok", failures);
  return failures ? 1 : 0;
}
