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
  c->device = dev;
  if (e == hipSuccess) e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) { c->last_hip = (int)e; delete c; return CAS_EHIP; }
  c->num_cu = v;
  e = hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
  if (e != hipSuccess) { c->last_hip = (int)e; delete c; return CAS_EHIP; }
  c->lds_max = v;
  // gfx950 lets a workgroup opt in to more LDS than the default limit
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeSharedMemPerBlockOptin, dev) == hipSuccess && v > c->lds_max)
    c->lds_max = v;
  (void)hipGetLastError();
  *out = c;
  return CAS_OK;
}

int cas_ctx_destroy(cas_ctx* ctx) {
  if (ctx) cas_prof_reset(ctx);
  delete ctx;
  return CAS_OK;
}

const char* cas_strerror(int code) {
  switch (code) {
    case CAS_OK: return "ok";
    case CAS_EINVAL: return "invalid argument (shape, alignment, format or NULL pointer)";
    case CAS_ENOTSUP: return "not supported by this build";
    case CAS_ENOMEM: return "workspace, pool or the library's fixed scratch array too small for this call";
    case CAS_EHIP: return "HIP call failed (see cas_last_hip_error)";
  }
  return "unknown error";
}

int cas_last_hip_error(const cas_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int cas_prof_enable(cas_ctx* ctx, int on) {
  if (!ctx) return CAS_EINVAL;
  ctx->prof_on = on != 0;
  return CAS_OK;
}

int cas_prof_read(cas_ctx* ctx, int kernel_class, int64_t* launches, double* total_ms, double* total_bytes) {
  if (!ctx || kernel_class < 0 || kernel_class >= cas::PROF_NCLASS || !launches || !total_ms || !total_bytes)
    return CAS_EINVAL;
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  *launches = 0; *total_ms = 0; *total_bytes = 0;
  for (const cas::ProfRec& r : ctx->prof) {
    if (r.cls != kernel_class) continue;
    float ms = 0.f;
    CAS_HIP(ctx, hipEventElapsedTime(&ms, r.e0, r.e1));
    *launches += 1; *total_ms += ms; *total_bytes += r.bytes;
  }
  return CAS_OK;
}

int cas_prof_reset(cas_ctx* ctx) {
  if (!ctx) return CAS_EINVAL;
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (cas::ProfRec& r : ctx->prof) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  ctx->prof.clear();
  return CAS_OK;
}

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
  if (!ctx || check_desc(desc) != CAS_OK || ld < desc->cols) return CAS_EINVAL;
  if (desc->rows == 0) return CAS_OK;  // nothing to encode; the pointers may be null
  if (!d_W || !d_spec || !d_verif) return CAS_EINVAL;
  if (!cas::aligned256(d_spec) || !cas::aligned256(d_verif)) return CAS_EINVAL;
  return cas::launch_encode_weight(ctx, d_W, ld, d_act_norm, *desc, d_spec, d_verif);
}

int cas_decode_weight(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, const void* d_verif, uint16_t* d_out,
                      int64_t ld) {
  if (!ctx || check_desc(desc) != CAS_OK || ld < desc->cols) return CAS_EINVAL;
  if (desc->rows == 0) return CAS_OK;
  if (!d_spec || !d_out) return CAS_EINVAL;
  if (!cas::aligned256(d_spec) || !cas::aligned256(d_verif)) return CAS_EINVAL;
  return cas::launch_decode_weight(ctx, *desc, d_spec, d_verif, d_out, ld);
}

int cas_gemv_draft(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, const uint16_t* d_x, int batch,
                   float* d_y) {
  if (!ctx || check_desc(desc) != CAS_OK || batch < 1 || batch > 4) return CAS_EINVAL;
  if (desc->rows == 0) return CAS_OK;  // empty output
  if (!d_spec || !d_x || !d_y || !cas::aligned256(d_spec)) return CAS_EINVAL;
  return cas::launch_gemv_draft(ctx, *desc, d_spec, d_x, batch, d_y);
}

int cas_gemv_draft_fused(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, const uint16_t* d_x, int batch,
                         float* d_y, const uint16_t* d_gain, float eps, int epilogue, uint16_t* d_out16) {
  if (!ctx || check_desc(desc) != CAS_OK || batch < 1 || batch > 4 || epilogue < 0 || epilogue > 2) return CAS_EINVAL;
  if (desc->rows == 0) return CAS_OK;
  if (!d_spec || !d_x || !cas::aligned256(d_spec)) return CAS_EINVAL;
  if ((epilogue == 0 && !d_y) || (epilogue != 0 && !d_out16)) return CAS_EINVAL;
  return cas::launch_gemv_draft_fused(ctx, *desc, d_spec, d_x, batch, d_y, d_gain, eps, epilogue, d_out16);
}

int cas_gemm_verify(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, const void* d_verif,
                    const uint16_t* d_X, int ncols, float* d_Y) {
  if (!ctx || check_desc(desc) != CAS_OK || ncols < 1 || ncols > 32) return CAS_EINVAL;
  if (desc->rows == 0) return CAS_OK;
  if (!d_spec || !d_verif || !d_X || !d_Y) return CAS_EINVAL;
  if (!cas::aligned256(d_spec) || !cas::aligned256(d_verif)) return CAS_EINVAL;
  return cas::launch_gemm_verify(ctx, *desc, d_spec, d_verif, d_X, ncols, d_Y);
}

int cas_kv_desc_init(cas_kv_desc* d) {
  if (!d) return CAS_EINVAL;
  if (d->head_dim != 128 || d->page_tokens != 64) return CAS_ENOTSUP;
  if (d->n_layers < 1 || d->n_kv_heads < 1 || d->n_pages < 1 || d->max_seqs < 1 || d->max_pages_per_seq < 1)
    return CAS_EINVAL;
  if (d->fmt.trunc_bits < 0 || d->fmt.trunc_bits > 7 || d->fmt.keep_permille < 0 || d->fmt.keep_permille > 1000)
    return CAS_EINVAL;
  if (d->fmt.exp_mode != CAS_EXP_RAW && d->fmt.exp_mode != CAS_EXP_SHARED) return CAS_ENOTSUP;
  const bool mx = d->fmt.exp_mode == CAS_EXP_SHARED;
  const int t = d->fmt.trunc_bits;
  int64_t K = ((int64_t)d->fmt.keep_permille * d->head_dim + 500) / 1000;
  K = std::max<int64_t>(0, std::min<int64_t>(d->head_dim, K));
  d->K = (int32_t)K;
  d->sw = (int32_t)words(K * (mx ? 9 - t : 16 - t));
  d->lw = (int32_t)words(K * t);
  d->pw = (int32_t)words((d->head_dim - K) * 16);
  d->tile_spec_bytes = up256((int64_t)d->page_tokens * (4 + (mx ? 1 : 0) + d->sw) * 4);
  d->tile_verif_bytes = up256((int64_t)d->page_tokens * (d->lw + d->pw) * 4);
  const int64_t tiles = (int64_t)d->n_layers * d->n_pages * 2 * d->n_kv_heads;
  d->spec_pool_bytes = tiles * d->tile_spec_bytes + kSlack;
  d->verif_pool_bytes = tiles * d->tile_verif_bytes + kSlack;
  return CAS_OK;
}

int cas_kv_create(const cas_kv_desc* desc, void* d_spec_pool, void* d_verif_pool, const int32_t* d_page_table,
                  cas_kv** out) {
  if (!desc || !d_spec_pool || !d_verif_pool || !d_page_table || !out) return CAS_EINVAL;
  cas_kv_desc chk = *desc;
  int rc = cas_kv_desc_init(&chk);
  if (rc != CAS_OK) return rc;
  if (chk.spec_pool_bytes != desc->spec_pool_bytes || chk.verif_pool_bytes != desc->verif_pool_bytes) return CAS_EINVAL;
  if (!cas::aligned256(d_spec_pool) || !cas::aligned256(d_verif_pool)) return CAS_EINVAL;
  cas_kv* kv = new (std::nothrow) cas_kv();
  if (!kv) return CAS_ENOMEM;
  kv->desc = chk;
  cas::KvGeom& g = kv->geom;
  g.n_layers = chk.n_layers; g.n_kv_heads = chk.n_kv_heads; g.page_tokens = chk.page_tokens;
  g.n_pages = chk.n_pages; g.max_pages_per_seq = chk.max_pages_per_seq;
  g.K = chk.K; g.t = chk.fmt.trunc_bits; g.sw = chk.sw; g.lw = chk.lw; g.pw = chk.pw;
  g.mx = chk.fmt.exp_mode == CAS_EXP_SHARED ? 1 : 0;
  g.spec_off = chk.page_tokens * (g.mx ? 5 : 4);
  g.tile_spec_words = (int)(chk.tile_spec_bytes / 4);
  g.tile_verif_words = (int)(chk.tile_verif_bytes / 4);
  kv->d_spec = d_spec_pool; kv->d_verif = d_verif_pool; kv->d_page_table = d_page_table;
  kv->h_len = new (std::nothrow) int32_t[chk.max_seqs]();
  if (!kv->h_len) { delete kv; return CAS_ENOMEM; }
  *out = kv;
  return CAS_OK;
}

int cas_kv_destroy(cas_kv* kv) {
  if (kv) { delete[] kv->h_len; delete kv; }
  return CAS_OK;
}

static int check_seq(const cas_kv* kv, int layer, int seq) {
  if (!kv || seq < 0 || seq >= kv->desc.max_seqs || layer < 0 || layer >= kv->desc.n_layers) return CAS_EINVAL;
  return CAS_OK;
}

int cas_kv_append(cas_ctx* ctx, cas_kv* kv, int layer, int seq, const uint16_t* d_K, const uint16_t* d_V, int n_tok) {
  if (!ctx || n_tok < 0 || check_seq(kv, layer, seq) != CAS_OK) return CAS_EINVAL;
  if (n_tok == 0) return CAS_OK;
  if (!d_K || !d_V) return CAS_EINVAL;
  const int64_t cap = (int64_t)kv->desc.max_pages_per_seq * kv->desc.page_tokens;
  if ((int64_t)kv->h_len[seq] + n_tok > cap) return CAS_ENOMEM;
  return cas::launch_kv_append(ctx, kv, layer, seq, d_K, d_V, n_tok, kv->h_len[seq]);
}

int cas_kv_set_len(cas_kv* kv, int seq, int32_t len) {
  if (check_seq(kv, 0, seq) != CAS_OK || len < 0) return CAS_EINVAL;
  if ((int64_t)len > (int64_t)kv->desc.max_pages_per_seq * kv->desc.page_tokens) return CAS_ENOMEM;
  kv->h_len[seq] = len;
  return CAS_OK;
}

int cas_kv_len(const cas_kv* kv, int seq, int32_t* len) {
  if (check_seq(kv, 0, seq) != CAS_OK || !len) return CAS_EINVAL;
  *len = kv->h_len[seq];
  return CAS_OK;
}

int cas_kv_read(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int pos0, int n_tok, int full, uint16_t* d_K,
                uint16_t* d_V) {
  if (!ctx || n_tok < 0 || pos0 < 0 || check_seq(kv, layer, seq) != CAS_OK) return CAS_EINVAL;
  if (n_tok == 0) return CAS_OK;
  if (!d_K || !d_V) return CAS_EINVAL;
  if ((int64_t)pos0 + n_tok > (int64_t)kv->desc.max_pages_per_seq * kv->desc.page_tokens) return CAS_EINVAL;
  return cas::launch_kv_read(ctx, kv, layer, seq, pos0, n_tok, full, d_K, d_V);
}

static int attention_call(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int full, const uint16_t* d_Q, int ncols,
                          int n_q_heads, const uint16_t* d_Knew, const uint16_t* d_Vnew, int n_new, uint16_t* d_O,
                          cas::AttnCall* c) {
  if (!ctx || !d_Q || !d_Knew || !d_Vnew || !d_O || check_seq(kv, layer, seq) != CAS_OK) return CAS_EINVAL;
  if (ncols < 1 || n_new < ncols || n_new > 64 || n_q_heads < kv->desc.n_kv_heads ||
      n_q_heads % kv->desc.n_kv_heads != 0)
    return CAS_EINVAL;
  if (ncols * (n_q_heads / kv->desc.n_kv_heads) > (full ? 80 : 48) || ncols > 16) return CAS_EINVAL;
  c->layer = layer; c->seq = seq; c->full = full ? 1 : 0;
  c->Q = d_Q; c->ncols = ncols; c->n_q_heads = n_q_heads;
  c->Knew = d_Knew; c->Vnew = d_Vnew; c->n_new = n_new; c->O = d_O;
  return CAS_OK;
}

int cas_attention(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int full, const uint16_t* d_Q, int ncols,
                  int n_q_heads, const uint16_t* d_Knew, const uint16_t* d_Vnew, int n_new, uint16_t* d_O) {
  cas::AttnCall c;
  const int rc = attention_call(ctx, kv, layer, seq, full, d_Q, ncols, n_q_heads, d_Knew, d_Vnew, n_new, d_O, &c);
  return rc != CAS_OK ? rc : cas::launch_attention(ctx, kv, c);
}

int cas_attention_static(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int full, const uint16_t* d_Q, int ncols,
                         int n_q_heads, const uint16_t* d_Knew, const uint16_t* d_Vnew, int n_new, uint16_t* d_O) {
  cas::AttnCall c;
  const int rc = attention_call(ctx, kv, layer, seq, full, d_Q, ncols, n_q_heads, d_Knew, d_Vnew, n_new, d_O, &c);
  return rc != CAS_OK ? rc : cas::launch_attention_static(ctx, kv, c);
}

size_t cas_attention_static_capacity(void) { return cas::attention_static_capacity(); }

int cas_attention_multi(cas_ctx* ctx, cas_kv* kv, int layer, int n_seqs, const int32_t* h_seqs, int full,
                        const uint16_t* const* h_d_Q, const int32_t* h_ncols, int n_q_heads,
                        const uint16_t* const* h_d_Knew, const uint16_t* const* h_d_Vnew, const int32_t* h_n_new,
                        uint16_t* const* h_d_O) {
  if (n_seqs < 1 || n_seqs > 16 || !h_seqs || !h_d_Q || !h_ncols || !h_d_Knew || !h_d_Vnew || !h_n_new || !h_d_O)
    return CAS_EINVAL;
  cas::AttnCall calls[16];
  for (int i = 0; i < n_seqs; ++i) {
    for (int j = 0; j < i; ++j)
      if (h_seqs[j] == h_seqs[i]) return CAS_EINVAL;
    const int rc = attention_call(ctx, kv, layer, h_seqs[i], full, h_d_Q[i], h_ncols[i], n_q_heads, h_d_Knew[i],
                                  h_d_Vnew[i], h_n_new[i], h_d_O[i], &calls[i]);
    if (rc != CAS_OK) return rc;
  }
  return cas::launch_attention_batch(ctx, kv, calls, n_seqs);
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

int cas_accept_sampling(const double* h_p, const double* h_q, const double* h_r, int gamma, int32_t* n_accepted) {
  if (gamma < 0 || !n_accepted || (gamma > 0 && (!h_p || !h_q || !h_r))) return CAS_EINVAL;
  int n = gamma;
  for (int i = 1; i <= gamma; ++i) {
    if (!(h_q[i - 1] > 0.0)) return CAS_EINVAL;
    if (h_r[i - 1] > h_p[i - 1] / h_q[i - 1]) {
      n = i - 1;
      break;
    }
  }
  *n_accepted = n;
  return CAS_OK;
}

int cas_objective(double alpha, double s_w, int w_keep_permille, int w_trunc_bits, double s_kv,
                  int kv_keep_permille, int kv_trunc_bits, int b_bits, double* h_j) {
  if (!h_j || !(alpha >= 0.0) || !(s_w >= 0.0) || !(s_kv >= 0.0) || b_bits < 1) return CAS_EINVAL;
  if (w_keep_permille < 0 || w_keep_permille > 1000 || kv_keep_permille < 0 || kv_keep_permille > 1000)
    return CAS_EINVAL;
  if (w_trunc_bits < 0 || w_trunc_bits > b_bits || kv_trunc_bits < 0 || kv_trunc_bits > b_bits) return CAS_EINVAL;
  const double den = s_w * (w_keep_permille / 1000.0) * (double)(b_bits - w_trunc_bits) +
                     s_kv * (kv_keep_permille / 1000.0) * (double)(b_bits - kv_trunc_bits);
  if (!(den > 0.0)) return CAS_EINVAL;
  *h_j = alpha / den;
  return CAS_OK;
}

int cas_tune_grid(const double* h_alpha, int n_keep, const int32_t* h_keep_permille, int n_trunc,
                  const int32_t* h_trunc_bits, double s_w, double s_kv, int kv_keep_permille, int kv_trunc_bits,
                  int b_bits, int32_t* best_keep_index, int32_t* best_trunc_index) {
  if (!h_alpha || !h_keep_permille || !h_trunc_bits || !best_keep_index || !best_trunc_index || n_keep < 1 ||
      n_trunc < 1)
    return CAS_EINVAL;
  double best = -1.0;
  for (int i = 0; i < n_keep; ++i) {
    for (int j = 0; j < n_trunc; ++j) {
      double v;
      int rc = cas_objective(h_alpha[(size_t)i * n_trunc + j], s_w, h_keep_permille[i], h_trunc_bits[j], s_kv,
                             kv_keep_permille, kv_trunc_bits, b_bits, &v);
      if (rc != CAS_OK) return rc;
      if (v > best) {
        best = v;
        *best_keep_index = i;
        *best_trunc_index = j;
      }
    }
  }
  return CAS_OK;
}

static double expected_tokens(double alpha, int gamma) {
  double n = 0.0, a = 1.0;  // 1 + alpha + ... + alpha^gamma
  for (int i = 0; i <= gamma; ++i) {
    n += a;
    a *= alpha;
  }
  return n;
}

int cas_speed_model(double alpha, int gamma, double t_draft, double t_verify, double t_plain, double* tokens_per_round,
                    double* tokens_per_s, double* speedup) {
  if (!(alpha >= 0.0) || !(alpha <= 1.0) || gamma < 0 || !(t_draft >= 0.0) || !(t_verify > 0.0) || !(t_plain >= 0.0))
    return CAS_EINVAL;
  const double n = expected_tokens(alpha, gamma);
  const double rate = n / ((double)gamma * t_draft + t_verify);
  if (tokens_per_round) *tokens_per_round = n;
  if (tokens_per_s) *tokens_per_s = rate;
  if (speedup) *speedup = rate * t_plain;
  return CAS_OK;
}

int cas_tune_measured(const double* h_alpha, const double* h_t_draft, const double* h_t_verify, int n_keep, int n_trunc,
                      int gamma, int32_t* best_keep_index, int32_t* best_trunc_index, double* h_tokens_per_s) {
  if (!h_alpha || !h_t_draft || !h_t_verify || !best_keep_index || !best_trunc_index || n_keep < 1 || n_trunc < 1)
    return CAS_EINVAL;
  double best = -1.0;
  for (int i = 0; i < n_keep; ++i) {
    for (int j = 0; j < n_trunc; ++j) {
      const size_t e = (size_t)i * n_trunc + j;
      double rate;
      const int rc = cas_speed_model(h_alpha[e], gamma, h_t_draft[e], h_t_verify[e], 0.0, nullptr, &rate, nullptr);
      if (rc != CAS_OK) return rc;
      if (h_tokens_per_s) h_tokens_per_s[e] = rate;
      if (rate > best) {
        best = rate;
        *best_keep_index = i;
        *best_trunc_index = j;
      }
    }
  }
  return CAS_OK;
}

}  // extern "C"
