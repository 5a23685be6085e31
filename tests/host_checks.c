/* Host-side exercise of the C ABI for sanitizer builds (plain C: also shows that the header is valid C).
 * Every call here must be answered by the library's host code alone - argument validation, shape checks and
 * workspace sizing - before any device work, so the program runs without a GPU.  tests/test_host_sanitizers.py
 * links it against a build of the library whose host code carries AddressSanitizer and
 * UndefinedBehaviorSanitizer instrumentation.  Device pointers are made-up non-null addresses: a correct
 * library never dereferences them on the host. */
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "moespec.h"

static int failures = 0;

#define EXPECT(cond)                                                   \
  do {                                                                 \
    if (!(cond)) {                                                     \
      fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      ++failures;                                                      \
    }                                                                  \
  } while (0)

static void *fake(uintptr_t a) { return (void *)a; }

static moespec_desc make_desc(int d, int n, int k, int f, int dtype) {
  moespec_desc ds;
  memset(&ds, 0, sizeof ds);
  ds.d = d;
  ds.n_experts = n;
  ds.top_k = k;
  ds.d_ff = f;
  ds.dtype = dtype;
  ds.renorm = 1;
  ds.gate = MOESPEC_GATE_SOFTMAX;
  return ds;
}

static void desc_and_workspace(void) {
  /* the five workload shapes and the larger trees */
  const int shapes[][6] = {{64, 8, 2, 96, MOESPEC_F32, 15},     {2048, 64, 8, 1024, MOESPEC_BF16, 63},
                           {2048, 64, 8, 1024, MOESPEC_BF16, 127}, {2048, 128, 8, 768, MOESPEC_BF16, 127},
                           {4096, 8, 2, 14336, MOESPEC_BF16, 63},  {2048, 64, 8, 1024, MOESPEC_BF16, 511}};
  size_t prev = 0;
  for (size_t i = 0; i < sizeof shapes / sizeof shapes[0]; ++i) {
    moespec_desc ds = make_desc(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4]);
    EXPECT(moespec_check_desc(&ds) == MOESPEC_OK);
    const size_t w = moespec_workspace_bytes(&ds, shapes[i][5]);
    EXPECT(w > 0);
    EXPECT(moespec_workspace_bytes(&ds, shapes[i][5] + 1) >= w);
    prev += w;
  }
  EXPECT(prev > 0);
  moespec_desc ds = make_desc(256, 16, 4, 256, MOESPEC_BF16);
  /* sizes at and beyond the supported range must not overflow the size arithmetic */
  const int32_t big[] = {1, 1024, 1025, 65535, 65536, 1 << 24, INT32_MAX, -1, INT32_MIN};
  for (size_t i = 0; i < sizeof big / sizeof big[0]; ++i) (void)moespec_workspace_bytes(&ds, big[i]);
  EXPECT(moespec_workspace_bytes(&ds, 0) == 0);
  EXPECT(moespec_workspace_bytes(NULL, 8) == 0);
  EXPECT(moespec_check_desc(NULL) == MOESPEC_ERR_INVALID_ARG);
  const int bad_fields[][5] = {{0, 16, 4, 256, MOESPEC_BF16},        {256, 0, 4, 256, MOESPEC_BF16},
                               {256, 16, 0, 256, MOESPEC_BF16},      {256, 16, 17, 256, MOESPEC_BF16},
                               {256, 16, 4, 0, MOESPEC_BF16},        {256, 16, 4, 256, 7},
                               {-256, 16, 4, 256, MOESPEC_BF16},     {256, -16, 4, 256, MOESPEC_BF16},
                               {INT32_MAX, 16, 4, 256, MOESPEC_BF16}, {256, INT32_MAX, 4, 256, MOESPEC_BF16},
                               {256, 16, 4, INT32_MAX, MOESPEC_BF16}, {250, 16, 4, 256, MOESPEC_BF16}};
  for (size_t i = 0; i < sizeof bad_fields / sizeof bad_fields[0]; ++i) {
    moespec_desc b = make_desc(bad_fields[i][0], bad_fields[i][1], bad_fields[i][2], bad_fields[i][3], bad_fields[i][4]);
    EXPECT(moespec_check_desc(&b) != MOESPEC_OK);
    EXPECT(moespec_workspace_bytes(&b, 63) == 0);
  }
  ds.gate = 2;
  EXPECT(moespec_check_desc(&ds) == MOESPEC_ERR_INVALID_ARG);
}

static void strings(void) {
  EXPECT(moespec_abi_version() > 0);
  for (int32_t st = -3; st < 12; ++st) {
    const char *s = moespec_status_string(st);
    EXPECT(s != NULL && strlen(s) > 0);
  }
  EXPECT(strcmp(moespec_status_string(MOESPEC_OK), "ok") == 0);
}

static void layer_calls(void) {
  moespec_desc ds = make_desc(256, 16, 4, 256, MOESPEC_BF16);
  moespec_weights w = {fake(0x40000), NULL, fake(0x50000), fake(0x60000), fake(0x70000)};
  void *h = fake(0x20000), *out = fake(0x30000), *ws = fake(0x100000);
  const size_t need = moespec_workspace_bytes(&ds, 8);
  EXPECT(need > 0);
  /* null and out-of-range arguments */
  EXPECT(moespec_layer_forward(NULL, &w, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, NULL, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, NULL, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, NULL, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, NULL, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, h, -1, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 0, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 17, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 2, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG); /* B < k under substitution */
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 8, 5, NULL, NULL, out, NULL, ws, need, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need - 1, NULL) ==
         MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(moespec_layer_forward(&ds, &w, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, 0, NULL) ==
         MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  moespec_weights w_missing = w;
  w_missing.w_down = NULL;
  EXPECT(moespec_layer_forward(&ds, &w_missing, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  /* the same checks guard the traced, the static-scratch and the stack entry points */
  EXPECT(moespec_layer_forward_traced(&ds, &w, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, NULL, NULL, NULL, ws, need,
                                      NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward_traced(&ds, &w, h, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL, NULL, ws, 1, NULL) ==
         MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(moespec_layer_forward_static(&ds, &w, NULL, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_layer_forward_static(&ds, &w, h, 8, 99, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  moespec_desc huge = make_desc(4096, 8, 2, 14336, MOESPEC_BF16);
  EXPECT(moespec_workspace_bytes(&huge, 1024) > MOESPEC_STATIC_SCRATCH_BYTES);
  EXPECT(moespec_layer_forward_static(&huge, &w, h, 1024, 4, MOESPEC_SUBSTITUTE, NULL, NULL, out, NULL) ==
         MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  moespec_weights layers[2] = {w, w};
  EXPECT(moespec_stack_forward(&ds, layers, 0, h, 8, 8, MOESPEC_SUBSTITUTE, 1, NULL, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_stack_forward(&ds, NULL, 2, h, 8, 8, MOESPEC_SUBSTITUTE, 1, NULL, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_stack_forward(&ds, layers, 2, NULL, 8, 8, MOESPEC_SUBSTITUTE, 1, NULL, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  layers[1].w_up = NULL;
  EXPECT(moespec_stack_forward(&ds, layers, 2, h, 8, 8, MOESPEC_SUBSTITUTE, 1, NULL, NULL, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_rms_scale(&ds, NULL, 8, out, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_rms_scale(&ds, h, -4, out, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_rms_scale(NULL, h, 8, out, NULL) == MOESPEC_ERR_INVALID_ARG);
}

static void stage_calls(void) {
  moespec_desc ds = make_desc(256, 16, 4, 256, MOESPEC_BF16);
  moespec_weights w = {fake(0x40000), NULL, fake(0x50000), fake(0x60000), fake(0x70000)};
  void *h = fake(0x20000), *out = fake(0x30000), *ws = fake(0x100000);
  double *probs = (double *)fake(0x200000);
  int32_t *ids = (int32_t *)fake(0x300000);
  float *wts = (float *)fake(0x400000);
  const size_t need = moespec_workspace_bytes(&ds, 8);
  EXPECT(moespec_route(&ds, &w, NULL, 8, probs, ids, wts, ws, need, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_route(&ds, &w, h, 0, probs, ids, wts, ws, need, NULL) != MOESPEC_ERR_HIP);
  EXPECT(moespec_route(&ds, &w, h, 8, probs, ids, wts, ws, 0, NULL) == MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(moespec_budget(&ds, NULL, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, ids, ids, wts, ids, ids, ids, NULL, ws, need,
                        NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_budget(&ds, probs, 8, 99, MOESPEC_SUBSTITUTE, NULL, NULL, ids, ids, wts, ids, ids, ids, NULL, ws, need,
                        NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_budget(&ds, probs, 8, 8, MOESPEC_SUBSTITUTE, NULL, NULL, ids, ids, wts, ids, ids, ids, NULL, ws, 0,
                        NULL) == MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(moespec_expert_ffn(&ds, &w, h, 8, 8, NULL, ids, ids, ids, wts, NULL, out, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_expert_ffn(&ds, &w, h, 8, -1, ids, ids, ids, ids, wts, NULL, out, ws, need, NULL) ==
         MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_expert_ffn(&ds, &w, h, 8, 8, ids, ids, ids, ids, wts, NULL, out, ws, 0, NULL) ==
         MOESPEC_ERR_WORKSPACE_TOO_SMALL);
}

static void analysis_calls(void) {
  moespec_desc ds = make_desc(256, 16, 4, 256, MOESPEC_BF16);
  moespec_weights w = {fake(0x40000), NULL, fake(0x50000), fake(0x60000), fake(0x70000)};
  void *h = fake(0x20000), *out = fake(0x30000), *ws = fake(0x100000);
  int32_t *ids = (int32_t *)fake(0x300000);
  int64_t *counts = (int64_t *)fake(0x500000);
  double *dbl = (double *)fake(0x600000);
  EXPECT(moespec_calibration_count(&ds, NULL, 8, counts, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_calibration_count(&ds, ids, 8, NULL, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_calibration_count(&ds, ids, -1, counts, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_static_shortlist(&ds, NULL, 4, ids, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_static_shortlist(&ds, counts, 0, ids, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_static_shortlist(&ds, counts, 17, ids, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_coverage_curve(&ds, NULL, dbl, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_coverage_curve(&ds, dbl, NULL, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_reconstruction_error(&ds, NULL, out, 8, dbl, ws, 1 << 20, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_reconstruction_error(&ds, out, out, 8, dbl, ws, 0, NULL) == MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(moespec_oracle_ranking(&ds, &w, NULL, 8, 8, ids, dbl, ws, 1 << 26, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_oracle_ranking(&ds, &w, h, 8, 0, ids, dbl, ws, 1 << 26, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_oracle_ranking(&ds, &w, h, 8, 8, ids, dbl, ws, 0, NULL) == MOESPEC_ERR_WORKSPACE_TOO_SMALL);
  EXPECT(moespec_stream_read(NULL, 1 << 20, (uint32_t *)ids, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_stream_read(h, 1 << 20, NULL, NULL) == MOESPEC_ERR_INVALID_ARG);
  EXPECT(moespec_stream_read(h, 12345, (uint32_t *)ids, NULL) == MOESPEC_ERR_INVALID_ARG);
}

int main(void) {
  strings();
  desc_and_workspace();
  layer_calls();
  stage_calls();
  analysis_calls();
  if (failures) {
    fprintf(stderr, "%d host check(s) failed\n", failures);
    return 1;
  }
  puts("host checks passed");
  return 0;
}
