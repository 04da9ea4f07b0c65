// Host-side internals of the library: context, error plumbing, kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/cassandra.h"

struct cas_ctx {
  hipStream_t stream;
  void* d_ws;
  size_t ws_bytes;
  int last_hip;
  int num_cu;
  int lds_max;  // bytes of LDS one workgroup may use
};

#define CAS_HIP(ctx, expr)                          \
  do {                                              \
    hipError_t e__ = (expr);                        \
    if (e__ != hipSuccess) {                        \
      (ctx)->last_hip = (int)e__;                   \
      return CAS_EHIP;                              \
    }                                               \
  } while (0)

namespace cas {
inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

int launch_encode_weight(cas_ctx*, const uint16_t* W, int64_t ld, const float* act, const cas_wdesc&, void* spec, void* verif);
int launch_decode_weight(cas_ctx*, const cas_wdesc&, const void* spec, const void* verif, uint16_t* out, int64_t ld);
int launch_gemv_draft(cas_ctx*, const cas_wdesc&, const void* spec, const uint16_t* x, int batch, float* y);
int launch_gemm_verify(cas_ctx*, const cas_wdesc&, const void* spec, const void* verif, const uint16_t* X, int ncols, float* Y);
}  // namespace cas
