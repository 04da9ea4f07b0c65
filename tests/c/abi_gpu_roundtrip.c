/* The library used from plain C with device memory from the HIP runtime (no Python, no torch):
 * encode a matrix, rebuild it exactly (Sec. 4.1 target view), and check the draft GEMV and the
 * verification GEMM against double-precision sums over the matrices the library itself
 * reconstructs (draft view / exact view).  Exit code 0 = all checks passed. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "cassandra.h"

#define CHECK(cond)                                              \
  do {                                                           \
    if (!(cond)) {                                               \
      fprintf(stderr, "line %d: %s\n", __LINE__, #cond);         \
      return 1;                                                  \
    }                                                            \
  } while (0)

static double bf16_value(uint16_t w) {
  uint32_t u = (uint32_t)w << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* deterministic bf16 patterns: sign, exponent 118..126, any mantissa (values below 1 in magnitude) */
static uint16_t pattern(uint32_t* state) {
  *state = *state * 1664525u + 1013904223u;
  {
    const uint32_t r = *state >> 8;
    return (uint16_t)(((r & 1u) << 15) | ((118u + (r >> 1) % 9u) << 7) | ((r >> 8) & 0x7Fu));
  }
}

int main(void) {
  enum { ROWS = 300, COLS = 2500, NC = 3 };
  cas_ctx* ctx = NULL;
  cas_fmt fmt;
  cas_wdesc d;
  uint16_t *hW, *hX, *hD, *hF;
  float *hy, *hY;
  void *dW, *dX, *dspec, *dverif, *dout, *dy;
  uint32_t seed = 12345u;
  size_t i;
  int r, c, k;

  memset(&fmt, 0, sizeof fmt);
  fmt.keep_permille = 600;
  fmt.trunc_bits = 4;
  CHECK(cas_weight_desc(ROWS, COLS, &fmt, &d) == CAS_OK);
  hW = (uint16_t*)malloc(sizeof(uint16_t) * ROWS * COLS);
  hD = (uint16_t*)malloc(sizeof(uint16_t) * ROWS * COLS);
  hF = (uint16_t*)malloc(sizeof(uint16_t) * ROWS * COLS);
  hX = (uint16_t*)malloc(sizeof(uint16_t) * NC * COLS);
  hy = (float*)malloc(sizeof(float) * ROWS);
  hY = (float*)malloc(sizeof(float) * NC * ROWS);
  CHECK(hW && hD && hF && hX && hy && hY);
  for (i = 0; i < (size_t)ROWS * COLS; ++i) hW[i] = pattern(&seed);
  for (i = 0; i < (size_t)NC * COLS; ++i) hX[i] = pattern(&seed);

  CHECK(hipMalloc(&dW, sizeof(uint16_t) * ROWS * COLS) == hipSuccess);
  CHECK(hipMalloc(&dX, sizeof(uint16_t) * NC * COLS) == hipSuccess);
  CHECK(hipMalloc(&dspec, (size_t)d.spec_bytes) == hipSuccess);
  CHECK(hipMalloc(&dverif, (size_t)d.verif_bytes) == hipSuccess);
  CHECK(hipMalloc(&dout, sizeof(uint16_t) * ROWS * COLS) == hipSuccess);
  CHECK(hipMalloc(&dy, sizeof(float) * NC * ROWS) == hipSuccess);
  CHECK(hipMemcpy(dW, hW, sizeof(uint16_t) * ROWS * COLS, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(hipMemcpy(dX, hX, sizeof(uint16_t) * NC * COLS, hipMemcpyHostToDevice) == hipSuccess);

  CHECK(cas_ctx_create(&ctx, NULL, NULL, 0) == CAS_OK);
  CHECK(cas_encode_weight(ctx, (const uint16_t*)dW, COLS, NULL, &d, dspec, dverif) == CAS_OK);
  /* exact view: the original matrix, bit for bit */
  CHECK(cas_decode_weight(ctx, &d, dspec, dverif, (uint16_t*)dout, COLS) == CAS_OK);
  CHECK(hipMemcpy(hF, dout, sizeof(uint16_t) * ROWS * COLS, hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(memcmp(hF, hW, sizeof(uint16_t) * ROWS * COLS) == 0);
  /* draft view: K values per row, each a bit prefix of the original word */
  CHECK(cas_decode_weight(ctx, &d, dspec, NULL, (uint16_t*)dout, COLS) == CAS_OK);
  CHECK(hipMemcpy(hD, dout, sizeof(uint16_t) * ROWS * COLS, hipMemcpyDeviceToHost) == hipSuccess);
  for (r = 0; r < ROWS; ++r) {
    int kept = 0;
    for (c = 0; c < COLS; ++c) {
      const uint16_t w = hW[(size_t)r * COLS + c], v = hD[(size_t)r * COLS + c];
      if (v != 0) {
        ++kept;
        CHECK(v == (uint16_t)(w & 0xFFF0u));
      }
    }
    CHECK(kept <= d.K && kept >= d.K - 8); /* a kept value whose leading bits are all zero reads as pruned */
  }
  CHECK(cas_gemv_draft(ctx, &d, dspec, (const uint16_t*)dX, 1, (float*)dy) == CAS_OK);
  CHECK(hipMemcpy(hy, dy, sizeof(float) * ROWS, hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(cas_gemm_verify(ctx, &d, dspec, dverif, (const uint16_t*)dX, NC, (float*)dy) == CAS_OK);
  CHECK(hipMemcpy(hY, dy, sizeof(float) * NC * ROWS, hipMemcpyDeviceToHost) == hipSuccess);
  for (r = 0; r < ROWS; ++r) {
    double wn = 0.0;
    for (c = 0; c < COLS; ++c) wn += bf16_value(hW[(size_t)r * COLS + c]) * bf16_value(hW[(size_t)r * COLS + c]);
    wn = sqrt(wn);
    for (k = 0; k < NC; ++k) {
      double ref = 0.0, dref = 0.0, xn = 0.0;
      for (c = 0; c < COLS; ++c) {
        const double x = bf16_value(hX[(size_t)k * COLS + c]);
        ref += bf16_value(hW[(size_t)r * COLS + c]) * x;
        dref += bf16_value(hD[(size_t)r * COLS + c]) * x;
        xn += x * x;
      }
      xn = sqrt(xn);
      CHECK(fabs((double)hY[(size_t)k * ROWS + r] - ref) <= 2e-5 * wn * xn);
      if (k == 0) CHECK(fabs((double)hy[r] - dref) <= 2e-5 * wn * xn);
    }
  }
  CHECK(cas_ctx_destroy(ctx) == CAS_OK);
  puts("abi gpu roundtrip ok");
  return 0;
}
