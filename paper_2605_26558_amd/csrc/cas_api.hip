// C ABI entry points: argument checks and dispatch to the kernel launchers.
#include <algorithm>
#include <new>
#include "cas_internal.hpp"

namespace {
inline int64_t words(int64_t bits) { return (bits + 31) / 32; }
inline int64_t up256(int64_t b) { return (b + 255) / 256 * 256; }
constexpr int64_t kSlack = 256;
}  // namespace

extern "C" {

int cas_ctx_create(cas_ctx** out, void* hip_stream, void* d_workspace, size_t ws_bytes) {
  if (!out) return CAS_EINVAL;
  cas_ctx* c = new (std::nothrow) cas_ctx();
  if (!c) return CAS_ENOMEM;
  c->stream = (hipStream_t)hip_stream;
  c->d_ws = d_workspace;
  c->ws_bytes = ws_bytes;
  c->last_hip = 0;
  int dev = 0, v = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) { c->last_hip = (int)e; delete c; return CAS_EHIP; }
  c->num_cu = v;
  e = hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
  if (e != hipSuccess) { c->last_hip = (int)e; delete c; return CAS_EHIP; }
  c->lds_max = v;
  *out = c;
  return CAS_OK;
}

int cas_ctx_destroy(cas_ctx* ctx) {
  delete ctx;
  return CAS_OK;
}

const char* cas_strerror(int code) {
  switch (code) {
    case CAS_OK: return "ok";
    case CAS_EINVAL: return "invalid argument (shape, alignment, format or NULL pointer)";
    case CAS_ENOTSUP: return "not supported by this build";
    case CAS_ENOMEM: return "workspace or pool too small";
    case CAS_EHIP: return "HIP call failed (see cas_last_hip_error)";
  }
  return "unknown error";
}

int cas_last_hip_error(const cas_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int cas_weight_desc(int64_t rows, int64_t cols, const cas_fmt* fmt, cas_wdesc* out) {
  if (!fmt || !out || rows < 0 || cols < 1 || cols > (1 << 20)) return CAS_EINVAL;
  if (fmt->trunc_bits < 0 || fmt->trunc_bits > 7) return CAS_EINVAL;
  if (fmt->keep_permille < 0 || fmt->keep_permille > 1000) return CAS_EINVAL;
  if (fmt->exp_mode != 0) return CAS_ENOTSUP;
  int64_t K = ((int64_t)fmt->keep_permille * cols + 500) / 1000;
  K = std::max<int64_t>(0, std::min<int64_t>(cols, K));
  const int t = fmt->trunc_bits;
  out->rows = rows; out->cols = cols; out->K = (int32_t)K; out->t = t;
  out->bw = (int32_t)words(cols);
  out->sw = (int32_t)words(K * (16 - t));
  out->lw = (int32_t)words(K * t);
  out->pw = (int32_t)words((cols - K) * 16);
  // per-matrix offsets stay below 2^32 so kernels can use 32-bit word offsets inside a row block
  if (rows * std::max<int64_t>(std::max(out->sw, out->pw), out->bw) * 4 > ((int64_t)1 << 40)) return CAS_EINVAL;
  out->off_bitmap = 0;
  out->off_spec = up256(rows * out->bw * 4);
  out->spec_bytes = up256(out->off_spec + rows * out->sw * 4 + kSlack);
  out->off_lo = 0;
  out->off_pruned = up256(rows * out->lw * 4 + kSlack);
  out->verif_bytes = up256(out->off_pruned + rows * out->pw * 4 + kSlack);
  return CAS_OK;
}

static int check_desc(const cas_wdesc* d) {
  if (!d || d->rows < 0 || d->cols < 1 || d->t < 0 || d->t > 7 || d->K < 0 || d->K > d->cols) return CAS_EINVAL;
  if (d->bw != words(d->cols) || d->sw != words((int64_t)d->K * (16 - d->t)) ||
      d->lw != words((int64_t)d->K * d->t) || d->pw != words((d->cols - d->K) * 16))
    return CAS_EINVAL;
  return CAS_OK;
}

int cas_encode_weight(cas_ctx* ctx, const uint16_t* d_W, int64_t ld, const float* d_act_norm, const cas_wdesc* desc,
                      void* d_spec, void* d_verif) {
  if (!ctx || !d_W || !d_spec || !d_verif || check_desc(desc) != CAS_OK || ld < desc->cols) return CAS_EINVAL;
  if (!cas::aligned256(d_spec) || !cas::aligned256(d_verif)) return CAS_EINVAL;
  return cas::launch_encode_weight(ctx, d_W, ld, d_act_norm, *desc, d_spec, d_verif);
}

int cas_decode_weight(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, const void* d_verif, uint16_t* d_out,
                      int64_t ld) {
  if (!ctx || !d_spec || !d_out || check_desc(desc) != CAS_OK || ld < desc->cols) return CAS_EINVAL;
  if (!cas::aligned256(d_spec) || !cas::aligned256(d_verif)) return CAS_EINVAL;
  return cas::launch_decode_weight(ctx, *desc, d_spec, d_verif, d_out, ld);
}

int cas_gemv_draft(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, const uint16_t* d_x, int batch,
                   float* d_y) {
  if (!ctx || !d_spec || !d_x || !d_y || check_desc(desc) != CAS_OK) return CAS_EINVAL;
  if (batch < 1 || batch > 4 || !cas::aligned256(d_spec)) return CAS_EINVAL;
  return cas::launch_gemv_draft(ctx, *desc, d_spec, d_x, batch, d_y);
}

int cas_gemm_verify(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, const void* d_verif,
                    const uint16_t* d_X, int ncols, float* d_Y) {
  if (!ctx || !d_spec || !d_verif || !d_X || !d_Y || check_desc(desc) != CAS_OK) return CAS_EINVAL;
  if (ncols < 1 || ncols > 16 || !cas::aligned256(d_spec) || !cas::aligned256(d_verif)) return CAS_EINVAL;
  return cas::launch_gemm_verify(ctx, *desc, d_spec, d_verif, d_X, ncols, d_Y);
}

int cas_accept(const int32_t* h_draft, const int32_t* h_target, int k, int32_t* n_accepted, int32_t* h_out) {
  if (k < 0 || !h_target || !n_accepted || !h_out || (k > 0 && !h_draft)) return CAS_EINVAL;
  int n = 0;
  while (n < k && h_draft[n] == h_target[n]) ++n;
  for (int i = 0; i < n; ++i) h_out[i] = h_draft[i];
  h_out[n] = h_target[n];
  *n_accepted = n;
  return CAS_OK;
}

}  // extern "C"
