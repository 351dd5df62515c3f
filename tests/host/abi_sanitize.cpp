// Host-side driver for the sanitizer build of the library (AddressSanitizer +
// UndefinedBehaviorSanitizer on the host code only): every call below must
// be decided on the host -- argument validation, the decode planner's integer
// arithmetic -- so it runs without a GPU.  Prints "ok" and exits 0 if every
// status is the expected one; a sanitizer report makes the process fail.
#include <climits>
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "qjl.h"

static int failures = 0;
#define EXPECT(cond)                                                         \
  do {                                                                       \
    if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

static qjl_shape shape(int b, int hq, int hkv, int n, int d, int m, int dt, float scale = 1.0f) {
  qjl_shape s;
  s.batch = b; s.q_heads = hq; s.kv_heads = hkv; s.n = n; s.d = d; s.m = m; s.dtype = dt; s.scale = scale;
  return s;
}

int main() {
  void* const P = reinterpret_cast<void*>(0x10000);      // aligned, never dereferenced: validation comes first
  void* const M = reinterpret_cast<void*>(0x10004);      // misaligned
  uint8_t* const P8 = static_cast<uint8_t*>(P);
  uint16_t* const P16 = static_cast<uint16_t*>(P);
  float* const PF = static_cast<float*>(P);
  int32_t* const PI = static_cast<int32_t*>(P);

  // ---- argument validation of every entry point
  const qjl_shape good = shape(1, 32, 8, 4096, 128, 256, QJL_BF16);
  EXPECT(qjl_version() >= 100);
  EXPECT(qjl_status_string(-99) != nullptr);
  EXPECT(qjl_make_sketch(1, 256, 128, QJL_BF16, nullptr, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_make_sketch(1, 0, 128, QJL_BF16, P, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_make_sketch(1, INT_MAX, INT_MAX, QJL_BF16, P, nullptr) == QJL_ERR_UNSUPPORTED);
  EXPECT(qjl_make_sketch_orthogonal(1, 256, 128, 9, P, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_quantize_keys(nullptr, P, P, P8, P16, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_quantize_keys(&good, M, P, P8, P16, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_project_query(&good, P, nullptr, PF, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_scores(&good, PF, P8, nullptr, PF, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_decode_attention(&good, P, P, P8, P16, P, PF, nullptr, 0, nullptr) == QJL_ERR_WORKSPACE);
  EXPECT(qjl_decode_attention(&good, P, P, P8, P16, P, PF, P, 16, nullptr) == QJL_ERR_WORKSPACE);
  EXPECT(qjl_decode_attention(&good, P, P, P8, P16, P, PF, M, size_t(1) << 30, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_decode_attention_splits(&good, 0, P, P, P8, P16, P, PF, P, size_t(1) << 30, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_decode_attention_noalloc(&good, P, P, P8, P16, nullptr, PF, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_decode_attention_dual(&good, 0, P, P, P8, P16, P16, P, PF, P, 1 << 20, nullptr, nullptr, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_decode_attention_dual(&good, 64, P, P, P8, P16, P16, P, PF, P, 1 << 20, nullptr, nullptr, nullptr) == QJL_ERR_UNSUPPORTED);
  EXPECT(qjl_decode_attention_vq(&good, 3, P, P, P8, P16, P8, P16, P16, PF, P, 1 << 20, nullptr, nullptr, nullptr) == QJL_ERR_UNSUPPORTED);
  EXPECT(qjl_decode_attention_dual_vq(&good, 128, 9, P, P, P8, P16, P16, P8, P16, P16, PF, P, 1 << 20, nullptr, nullptr, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_generation_step(&good, 128, 4, 4096, P, P, P, P, PI, 4, P8, P16, P16, P8, P16, P16, PF, P, 1 << 20, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_generation_step(&good, 128, 4, -1, P, P, P, P, PI, 4, P8, P16, P16, P8, P16, P16, PF, P, 1 << 20, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_generation_step(&good, 128, 4, 7, P, P, P, P, nullptr, 4, P8, P16, P16, P8, P16, P16, PF, P, 1 << 20, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_generation_step_devpos(&good, 128, 4, nullptr, P, P, P, P, PI, 4, P8, P16, P16, P8, P16, P16, PF, P, 1 << 20, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_generation_step_devpos(&good, 128, 4, PI, P, P, P, P, PI, 4, P8, P16, P16, P8, P16, P16, PF, P, 16, nullptr) == QJL_ERR_WORKSPACE);
  EXPECT(qjl_generation_step_devpos(&good, 128, 3, PI, P, P, P, P, PI, 4, P8, P16, P16, P8, P16, P16, PF, P, 1 << 20, nullptr) == QJL_ERR_UNSUPPORTED);
  EXPECT(qjl_select_outliers(&good, P, 17, PI, P, 1 << 20, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_select_outliers(&good, P, 4, PI, P, 0, nullptr) == QJL_ERR_WORKSPACE);
  EXPECT(qjl_make_dual_sketch(&good, 0, P, P, PI, 4, P, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_quantize_keys_dual(&good, 128, P, P, nullptr, 4, P8, P16, P16, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_quantize_values(&good, 0, P, P8, P16, P16, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_append_keys(&good, 4090, 7, P, P, P8, P16, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_append_keys(&good, INT_MAX, INT_MAX, P, P, P8, P16, nullptr) == QJL_ERR_INVALID_ARG);
  EXPECT(qjl_decode_step(&good, 4096, P, P, P, P8, P16, P, PF, P, 1 << 20, nullptr) == QJL_ERR_INVALID_ARG);
  // shapes at the edge of the integer ranges
  const qjl_shape huge = shape(INT_MAX, INT_MAX, INT_MAX, INT_MAX, 128, 256, QJL_BF16);
  EXPECT(qjl_quantize_keys(&huge, P, P, P8, P16, nullptr) == QJL_ERR_UNSUPPORTED);
  EXPECT(qjl_decode_workspace_bytes(&huge) == 0 || qjl_decode_workspace_bytes(&huge) > 0);   // must not overflow
  const qjl_shape bad[] = {shape(0, 32, 8, 64, 128, 256, QJL_BF16), shape(1, 32, 5, 64, 128, 256, QJL_BF16),
                           shape(1, 32, 8, 0, 128, 256, QJL_BF16), shape(1, 32, 8, 64, 128, 256, 3),
                           shape(1, 32, 8, 64, 128, 256, QJL_BF16, 0.0f / 0.0f), shape(-1, -1, -1, -1, -1, -1, -1)};
  for (const qjl_shape& s : bad) {
    EXPECT(qjl_decode_workspace_bytes(&s) == 0);
    EXPECT(qjl_decode_plan(&s, 0, 0, nullptr) == 0);
    EXPECT(qjl_outlier_workspace_bytes(&s) == 0);
    EXPECT(qjl_decode_attention(&s, P, P, P8, P16, P, PF, P, 1 << 20, nullptr) == QJL_ERR_INVALID_ARG);
  }

  // ---- the decode planner: integer arithmetic over the whole range of shapes
  const int ns[] = {1, 63, 64, 65, 511, 512, 513, 4095, 4096, 5000, 33000, 65283, 70000, 131072, 1 << 20, 1 << 27, INT_MAX};
  const int heads[][2] = {{1, 1}, {32, 32}, {32, 8}, {6, 2}, {3, 1}, {64, 1}, {4096, 512}};
  const int batches[] = {1, 4, 16, 4096, 1 << 20};
  const int splits[] = {0, 1, 2, 7, 64, 512, 513, 4096, INT_MAX};
  const int ms[][2] = {{128, 0}, {256, 0}, {512, 0}, {128, 128}, {256, 128}, {512, 128}, {256, 256}};
  long plans = 0;
  for (int n : ns) for (auto& h : heads) for (int b : batches) for (auto& mm : ms) for (int dt : {QJL_F32, QJL_BF16}) {
    const qjl_shape s = shape(b, h[0], h[1], n, 128, mm[0], dt);
    size_t last_auto = 0;
    for (int sp : splits) {
      int32_t out[3] = {0, 0, 0};
      const size_t total = qjl_decode_plan(&s, mm[1], sp, out);
      if ((long)b * h[1] * n > (1L << 40) || (long)b * h[0] > INT_MAX || n > (1 << 30)) { EXPECT(total == 0); continue; }   // documented limits
      EXPECT(total > 0);
      EXPECT(out[0] == 1 || out[0] == 2 || out[0] == 4);
      EXPECT(out[1] >= 1 && out[1] <= 512);
      if (!(out[2] >= 64 && out[2] % 64 == 0) && failures < 5)
        std::printf("plan b=%d hq=%d hkv=%d n=%d m=%d+%d dt=%d splits=%d -> gt=%d nsplit=%d chunk=%d\n", b, h[0], h[1], n, mm[0], mm[1], dt, sp, out[0], out[1], out[2]);
      EXPECT(out[2] >= 64 && out[2] % 64 == 0);
      EXPECT((long)out[1] * out[2] >= n && (long)(out[1] - 1) * out[2] < n);
      EXPECT(total >= (size_t)b * h[0] * out[1] * 132 * 4);
      if (sp == 0) last_auto = total;
      ++plans;
    }
    // the workspace of a capacity covers shorter contexts
    if (n > 1) {
      const qjl_shape shorter = shape(b, h[0], h[1], n / 2 + 1, 128, mm[0], dt);
      if ((long)b * h[1] * n <= (1L << 40) && (long)b * h[0] <= INT_MAX && n <= (1 << 30)) EXPECT(qjl_decode_plan(&shorter, mm[1], 0, nullptr) <= last_auto);
    }
  }
  EXPECT(qjl_decode_plan(&good, -1, 0, nullptr) == 0);
  EXPECT(qjl_decode_plan(&good, 0, -5, nullptr) == 0);
  EXPECT(qjl_decode_noalloc_max_bytes() == (size_t(4) << 20));
  std::printf("%ld plans checked\n", plans);
  if (failures) { std::printf("%d expectations failed\n", failures); return 1; }
  std::printf("ok\n");
  return 0;
}
