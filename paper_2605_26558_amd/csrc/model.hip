// Llama-3 style decoder around the Cassandra kernels (Fig. 2_1 structure): the small
// element-wise kernels between the linear layers and attention, and the draft / verify /
// commit sequence of one speculative round (Sec. 2.2, Sec. 4.1).  Every tensor that passes
// from one operation to the next is rounded to bf16; inside an operation arithmetic is fp32.
#include <algorithm>
#include <new>
#include <vector>
#include "cas_device.hpp"
#include "cas_internal.hpp"

struct cas_model {
  cas_model_cfg cfg;
  cas_layer_weights* layers;  // host copy
  cas_tensor lm_head;
  const uint16_t* d_embed;
  const uint16_t* d_g_final;
  const float* d_rope;
  // activation buffers (device, carved from the caller's block)
  uint16_t *h, *xn, *q, *ao, *act, *knew, *vnew;
  float *y, *logits;
  int32_t *tok, *tgt;  // token chain of a round: pending + drafts, and the target's tokens
  float* amax_v;       // per-slice argmax candidates
  int32_t* amax_i;
  // Linear layers switched to the unary form of their speculation data (cas_model_use_unary):
  // entry 4 * layer + {0 wqkv, 1 wo, 2 wgu, 3 wd}, the output head last.
  // or to the shared-exponent form of the tensor (cas_model_use_mx): then the converted matrix is the weight
  struct UnaryRef {
    bool on = false;   // unary form
    cas_udesc u;
    const void* d_uspec = nullptr;
    bool mx_on = false;  // shared-exponent form
    cas_mxdesc mx;
    const void* d_mxspec = nullptr;
    const void* d_mxverif = nullptr;
  };
  std::vector<UnaryRef> unary;
};

namespace cas {

__global__ __launch_bounds__(256) void embed_kernel(const int32_t* __restrict__ tok, const uint16_t* __restrict__ emb,
                                                    uint16_t* __restrict__ h, int hidden, int vocab) {
  const int c = blockIdx.x;
  int t = tok[c];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  for (int i = threadIdx.x; i < hidden; i += 256) h[(size_t)c * hidden + i] = emb[(size_t)t * hidden + i];
}

// xn = bf16(x * rsqrt(mean(x^2) + eps) * g), one workgroup per column.  A column of up to
// 8192 values (a multiple of 8) is read once with 16-byte loads, together with the gain, and
// stays in registers between the reduction and the scaling.
constexpr int kNormThreads = 512;
__global__ __launch_bounds__(kNormThreads) void rmsnorm_kernel(const uint16_t* __restrict__ h,
                                                               const uint16_t* __restrict__ g,
                                                               uint16_t* __restrict__ out, int n, float eps) {
  __shared__ float red[kNormThreads / 64];
  const int c = blockIdx.x, tid = threadIdx.x;
  const uint16_t* x = h + (size_t)c * n;
  uint16_t* o = out + (size_t)c * n;
  const bool fast = (n & 7) == 0 && n <= 2 * 8 * kNormThreads &&
                    ((reinterpret_cast<uintptr_t>(h) | reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(out)) & 15) == 0;
  uint4 xv[2], gv[2];
  float ss = 0.f;
  if (fast) {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int i = (tid + k * kNormThreads) * 8;
      xv[k] = gv[k] = make_uint4(0, 0, 0, 0);
      if (i < n) {
        xv[k] = *reinterpret_cast<const uint4*>(x + i);
        gv[k] = *reinterpret_cast<const uint4*>(g + i);
      }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const uint32_t w[4] = {xv[k].x, xv[k].y, xv[k].z, xv[k].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float lo = __uint_as_float(w[e] << 16), hi = __uint_as_float(w[e] & 0xFFFF0000u);
        ss += lo * lo;
        ss += hi * hi;
      }
    }
  } else {
    for (int i = tid; i < n; i += kNormThreads) {
      const float v = bf16_to_f32(x[i]);
      ss += v * v;
    }
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  ss = 0.f;
#pragma unroll
  for (int w = 0; w < kNormThreads / 64; ++w) ss += red[w];
  const float r = 1.0f / sqrtf(ss / (float)n + eps);
  if (fast) {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int i = (tid + k * kNormThreads) * 8;
      if (i < n) {
        const uint32_t w[4] = {xv[k].x, xv[k].y, xv[k].z, xv[k].w};
        const uint32_t gw[4] = {gv[k].x, gv[k].y, gv[k].z, gv[k].w};
        uint32_t ov[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = __uint_as_float(w[e] << 16) * r * __uint_as_float(gw[e] << 16);
          const float hi = __uint_as_float(w[e] & 0xFFFF0000u) * r * __uint_as_float(gw[e] & 0xFFFF0000u);
          ov[e] = (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
        }
        *reinterpret_cast<uint4*>(o + i) = make_uint4(ov[0], ov[1], ov[2], ov[3]);
      }
    }
  } else {
    for (int i = tid; i < n; i += kNormThreads) o[i] = f32_to_bf16(bf16_to_f32(x[i]) * r * bf16_to_f32(g[i]));
  }
}

// token = lowest index among the maxima of a logits row; stage 1: one candidate per slice
constexpr int kArgmaxSlices = 64;
__device__ __forceinline__ void argmax_fold(float& best, int& idx, float v, int i) {
  if (v > best || (v == best && i < idx)) { best = v; idx = i; }
}
__global__ __launch_bounds__(256) void argmax_part_kernel(const float* __restrict__ logits, int vocab,
                                                          float* __restrict__ pv, int32_t* __restrict__ pi) {
  __shared__ float bv[4];
  __shared__ int bi[4];
  const int c = blockIdx.y, sl = blockIdx.x;
  const int per = (vocab + kArgmaxSlices - 1) / kArgmaxSlices;
  const int lo = sl * per, hi = min(vocab, lo + per);
  const float* x = logits + (size_t)c * vocab;
  float best = -INFINITY;
  int idx = 0x7FFFFFFF;
  for (int i = lo + threadIdx.x; i < hi; i += 256) argmax_fold(best, idx, x[i], i);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) argmax_fold(best, idx, __shfl_xor(best, o, 64), __shfl_xor(idx, o, 64));
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = idx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) argmax_fold(best, idx, bv[w], bi[w]);
    pv[c * kArgmaxSlices + sl] = best;
    pi[c * kArgmaxSlices + sl] = idx;
  }
}
__global__ __launch_bounds__(64) void argmax_final_kernel(const float* __restrict__ pv, const int32_t* __restrict__ pi,
                                                          int32_t* __restrict__ out) {
  const int c = blockIdx.x;
  float best = pv[c * kArgmaxSlices + threadIdx.x];
  int idx = pi[c * kArgmaxSlices + threadIdx.x];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) argmax_fold(best, idx, __shfl_xor(best, o, 64), __shfl_xor(idx, o, 64));
  if (threadIdx.x == 0) out[c] = idx == 0x7FFFFFFF ? 0 : idx;
}

// Probability of one token under the softmax of a row of logits (p_i(x), q_i(x) of Eq. 1): one
// workgroup per row; maximum, then sum of exponentials, both reduced in a fixed order.
constexpr int kProbThreads = 1024;
__global__ __launch_bounds__(kProbThreads) void token_prob_kernel(const float* __restrict__ logits, int vocab,
                                                                  const int32_t* __restrict__ tokens,
                                                                  float* __restrict__ probs) {
  __shared__ float red[kProbThreads / 64];
  const float* x = logits + (size_t)blockIdx.x * vocab;
  const int tid = threadIdx.x;
  float mx = -INFINITY;
  for (int i = tid; i < vocab; i += kProbThreads) mx = fmaxf(mx, x[i]);
  mx = wave_max(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  mx = red[0];
#pragma unroll
  for (int w = 1; w < kProbThreads / 64; ++w) mx = fmaxf(mx, red[w]);
  __syncthreads();
  float sum = 0.f;
  for (int i = tid; i < vocab; i += kProbThreads) sum += expf(x[i] - mx);
  sum = wave_sum(sum);
  if ((tid & 63) == 0) red[tid >> 6] = sum;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < kProbThreads / 64; ++w) t += red[w];
    const int tok = tokens[blockIdx.x];
    probs[blockIdx.x] = (tok >= 0 && tok < vocab) ? expf(x[tok] - mx) / t : 0.f;
  }
}

// Glue of the plain bf16 baseline step (the encoded passes fuse these into their GEMV / GEMM
// launches): h = bf16(h + bf16(y)), and act[i] = bf16(silu(bf16(y[2i])) * bf16(y[2i+1])).
__global__ __launch_bounds__(256) void residual_add_kernel(uint16_t* __restrict__ h, const float* __restrict__ y, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) h[i] = f32_to_bf16(bf16_to_f32(h[i]) + round_bf16(y[i]));
}
__global__ __launch_bounds__(256) void swiglu_kernel(const float* __restrict__ y, uint16_t* __restrict__ act, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    const float g = round_bf16(y[2 * i]), u = round_bf16(y[2 * i + 1]);
    act[i] = f32_to_bf16(g / (1.0f + expf(-g)) * u);
  }
}

// tokens [steps][n_seqs] -> [n_seqs][steps]
__global__ void transpose_tokens_kernel(const int32_t* __restrict__ in, int32_t* __restrict__ out, int steps, int n_seqs) {
  const int i = threadIdx.x;
  if (i < steps * n_seqs) out[(i % n_seqs) * steps + i / n_seqs] = in[i];
}

#define CAS_TRY(expr)            \
  do {                           \
    int rc__ = (expr);           \
    if (rc__ != CAS_OK) return rc__; \
  } while (0)

// A run of consecutive columns that belong to one sequence.  slot0: index of the run's first
// column among the in-flight positions of the sequence (its position is len + slot0).
struct ColGroup {
  int seq, ncols, slot0;
};

static int model_seqs(const cas_model_cfg& c) { return c.max_seqs > 0 ? c.max_seqs : 1; }

// columns one sequence may contribute to a pass: what one attention call takes
static int seq_cols_max(const cas_model_cfg& c) {
  return std::min({(int)c.max_cols, 16, 80 / (c.n_q_heads / c.n_kv_heads)});
}

// Runs the columns of `ng` groups (token ids on the device, group after group) through the
// model in one pass: the linear layers see all columns at once, attention runs over each
// sequence's own cache and in-flight slots, four sequences per launch.
static int forward(cas_ctx* ctx, cas_model* m, cas_kv* kv, const ColGroup* grp, int ng, const int32_t* d_tokens,
                   bool full, int32_t* d_out, float* d_logits) {
  const cas_model_cfg& c = m->cfg;
  const int qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
  int ncols = 0;
  for (int i = 0; i < ng; ++i) {
    const ColGroup& g = grp[i];
    if (g.seq < 0 || g.seq >= kv->desc.max_seqs || g.seq >= model_seqs(c) || g.ncols < 1 || g.slot0 < 0)
      return CAS_EINVAL;
    if (g.ncols > seq_cols_max(c)) return CAS_EINVAL;
    if (kv->h_len[g.seq] + g.slot0 + g.ncols > c.max_pos || g.slot0 + g.ncols > c.max_cols) return CAS_EINVAL;
    for (int j = 0; j < i; ++j)
      if (grp[j].seq == g.seq) return CAS_EINVAL;  // one run per sequence and pass
    ncols += g.ncols;
  }
  if (ncols < 1 || ncols > c.max_cols || (!full && ncols > 4)) return CAS_EINVAL;
  hipStream_t st = ctx->stream;
  float* logits = d_logits ? d_logits : m->logits;
  // A linear layer of the draft pass.  Raw form: one fused launch (norm of x, product, residual
  // add or SwiGLU).  Unary form: the same operations with the same roundings as separate
  // launches around the GEMV that reads the unary buffer, column by column.
  auto lin_draft = [&](const cas_tensor& T, const cas_model::UnaryRef& U, const uint16_t* x, float* y,
                       const uint16_t* gain, int epi, uint16_t* out16) -> int {
    const int rows = (int)T.desc.rows, cols = (int)T.desc.cols;
    if (U.mx_on) {  // the kernel of the raw form with the shared-exponent field decode, one column per launch
      for (int col = 0; col < ncols; ++col) {
        const int rc = launch_gemv_draft_mx_fused(ctx, U.mx, U.d_mxspec, x + (size_t)col * cols,
                                                  y ? y + (size_t)col * rows : nullptr, gain, c.rms_eps, epi,
                                                  out16 ? out16 + (size_t)col * (epi == 2 ? rows / 2 : rows) : nullptr);
        if (rc != CAS_OK) return rc;
      }
      return CAS_OK;
    }
    if (!U.on) return launch_gemv_draft_fused(ctx, T.desc, T.d_spec, x, ncols, y, gain, c.rms_eps, epi, out16);
    if (gain) {
      hipLaunchKernelGGL(rmsnorm_kernel, dim3(ncols), dim3(kNormThreads), 0, st, x, gain, m->xn, cols, c.rms_eps);
      x = m->xn;
    }
    float* yy = epi == 0 ? y : m->y;
    for (int col = 0; col < ncols; ++col) {
      const int rc = cas_gemv_draft_unary(ctx, &U.u, U.d_uspec, x + (size_t)col * cols, yy + (size_t)col * rows);
      if (rc != CAS_OK) return rc;
    }
    if (epi == 1) {
      const int n = ncols * rows;
      hipLaunchKernelGGL(residual_add_kernel, dim3((n + 255) / 256), dim3(256), 0, st, out16, yy, n);
    } else if (epi == 2) {
      const int n = ncols * (rows / 2);
      hipLaunchKernelGGL(swiglu_kernel, dim3((n + 255) / 256), dim3(256), 0, st, yy, out16, n);
    }
    return CAS_OK;
  };
  // ... and of the verification pass: the unary form goes through the same kernel after its
  // rows are re-coded, so both forms give the same bits.
  auto lin_verify = [&](const cas_tensor& T, const cas_model::UnaryRef& U, const uint16_t* X, float* Y, int epi,
                        uint16_t* out16) -> int {
    if (U.mx_on) return launch_gemm_verify_mx_fused(ctx, U.mx, U.d_mxspec, U.d_mxverif, X, ncols, Y, epi, out16);
    if (!U.on) return launch_gemm_verify_fused(ctx, T.desc, T.d_spec, T.d_verif, X, ncols, Y, epi, out16);
    return launch_gemm_verify_unary_fused(ctx, U.u, U.d_uspec, T.d_verif, X, ncols, Y, epi, out16);
  };
  hipLaunchKernelGGL(embed_kernel, dim3(ncols), dim3(256), 0, st, d_tokens, m->d_embed, m->h, c.hidden, c.vocab);
  for (int l = 0; l < c.n_layers; ++l) {
    const cas_layer_weights& L = m->layers[l];
    const cas_model::UnaryRef* UL = &m->unary[4 * (size_t)l];
    // the draft pass fuses the norms, residual adds and SwiGLU into its GEMV launches
    if (full) {
      hipLaunchKernelGGL(rmsnorm_kernel, dim3(ncols), dim3(kNormThreads), 0, st, m->h, L.d_g_attn, m->xn, c.hidden, c.rms_eps);
      CAS_TRY(lin_verify(L.wqkv, UL[0], m->xn, m->y, 0, nullptr));
    } else {
      CAS_TRY(lin_draft(L.wqkv, UL[0], m->h, m->y, L.d_g_attn, 0, nullptr));
    }
    // the attention kernel splits the projection itself: bf16 rounding, rotary embedding of q and
    // k, and the copy of this pass's k, v into their in-flight slots
    AttnCall calls[16];
    for (int i = 0, c0 = 0; i < ng; c0 += grp[i].ncols, ++i) {
      const ColGroup& g = grp[i];
      const size_t slots = ((size_t)g.seq * c.n_layers + l) * c.max_cols * kvd;  // in-flight K/V of (sequence, layer)
      AttnCall& ac = calls[i];
      ac.layer = l; ac.seq = g.seq; ac.full = full ? 1 : 0;
      ac.Q = m->q; ac.ncols = g.ncols; ac.n_q_heads = c.n_q_heads;
      ac.Knew = m->knew + slots; ac.Vnew = m->vnew + slots; ac.n_new = g.slot0 + g.ncols;
      ac.O = m->ao + (size_t)c0 * qd;
      ac.qkv = m->y + (size_t)c0 * (qd + 2 * kvd); ac.ystride = qd + 2 * kvd; ac.slot0 = g.slot0; ac.rope = m->d_rope;
      ac.Kslot = m->knew + slots; ac.Vslot = m->vnew + slots;
    }
    CAS_TRY(launch_attention_batch(ctx, kv, calls, ng));
    if (full) {
      // residual adds and SwiGLU ride in the epilogue of the verification GEMM
      CAS_TRY(lin_verify(L.wo, UL[1], m->ao, nullptr, 1, m->h));
      hipLaunchKernelGGL(rmsnorm_kernel, dim3(ncols), dim3(kNormThreads), 0, st, m->h, L.d_g_ffn, m->xn, c.hidden, c.rms_eps);
      CAS_TRY(lin_verify(L.wgu, UL[2], m->xn, nullptr, 2, m->act));
      CAS_TRY(lin_verify(L.wd, UL[3], m->act, nullptr, 1, m->h));
    } else {
      CAS_TRY(lin_draft(L.wo, UL[1], m->ao, nullptr, nullptr, 1, m->h));
      CAS_TRY(lin_draft(L.wgu, UL[2], m->h, nullptr, L.d_g_ffn, 2, m->act));
      CAS_TRY(lin_draft(L.wd, UL[3], m->act, nullptr, nullptr, 1, m->h));
    }
  }
  if (full) {
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(ncols), dim3(kNormThreads), 0, st, m->h, m->d_g_final, m->xn, c.hidden, c.rms_eps);
    CAS_TRY(lin_verify(m->lm_head, m->unary.back(), m->xn, logits, 0, nullptr));
  } else {
    CAS_TRY(lin_draft(m->lm_head, m->unary.back(), m->h, logits, m->d_g_final, 0, nullptr));
  }
  if (d_out) {
    hipLaunchKernelGGL(argmax_part_kernel, dim3(kArgmaxSlices, ncols), dim3(256), 0, st, logits, c.vocab, m->amax_v,
                       m->amax_i);
    hipLaunchKernelGGL(argmax_final_kernel, dim3(ncols), dim3(64), 0, st, m->amax_v, m->amax_i, d_out);
  }
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

static size_t carve(size_t& off, size_t bytes) {
  size_t o = off;
  off = (off + bytes + 255) / 256 * 256;
  return o;
}

struct ActLayout {
  size_t h, xn, q, ao, act, knew, vnew, y, logits, tok, tgt, amax_v, amax_i, total;
};

static ActLayout act_layout(const cas_model_cfg& c) {
  const size_t nc = c.max_cols, qd = (size_t)c.n_q_heads * c.head_dim, kvd = (size_t)c.n_kv_heads * c.head_dim;
  const size_t ymax = std::max<size_t>({qd + 2 * kvd, 2 * (size_t)c.ffn, (size_t)c.hidden});
  ActLayout L;
  size_t off = 0;
  L.h = carve(off, nc * c.hidden * 2);
  L.xn = carve(off, nc * std::max<size_t>(c.hidden, qd) * 2);
  L.q = carve(off, nc * qd * 2);
  L.ao = carve(off, nc * qd * 2);
  L.act = carve(off, nc * c.ffn * 2);
  L.knew = carve(off, (size_t)model_seqs(c) * c.n_layers * nc * kvd * 2);
  L.vnew = carve(off, (size_t)model_seqs(c) * c.n_layers * nc * kvd * 2);
  L.y = carve(off, nc * ymax * 4);
  L.logits = carve(off, nc * (size_t)c.vocab * 4);
  L.tok = carve(off, 8 * nc * 4);        // draft tokens of up to 4 sequences step-major, then sequence-major

  L.tgt = carve(off, 4 * nc * 4);
  L.amax_v = carve(off, nc * kArgmaxSlices * 4);
  L.amax_i = carve(off, nc * kArgmaxSlices * 4);
  L.total = off;
  return L;
}

static int check_cfg(const cas_model_cfg* c) {
  if (!c || c->hidden < 1 || c->n_layers < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->ffn < 1 || c->vocab < 1)
    return CAS_EINVAL;
  if (c->head_dim != 128) return CAS_ENOTSUP;
  if (c->n_q_heads % c->n_kv_heads != 0 || c->max_cols < 1 || c->max_cols > 32 || c->max_pos < 1) return CAS_EINVAL;
  if (c->max_seqs < 0 || c->max_seqs > 64) return CAS_EINVAL;
  if (c->n_q_heads / c->n_kv_heads > 48) return CAS_EINVAL;
  return CAS_OK;
}

}  // namespace cas

extern "C" {

int cas_model_act_bytes(const cas_model_cfg* cfg, size_t* bytes) {
  if (!bytes) return CAS_EINVAL;
  int rc = cas::check_cfg(cfg);
  if (rc != CAS_OK) return rc;
  *bytes = cas::act_layout(*cfg).total;
  return CAS_OK;
}

int cas_model_create(const cas_model_cfg* cfg, const cas_model_weights* w, void* d_act, size_t act_bytes,
                     cas_model** out) {
  if (!w || !d_act || !out || !w->layers || !w->d_embed || !w->d_g_final || !w->d_rope) return CAS_EINVAL;
  int rc = cas::check_cfg(cfg);
  if (rc != CAS_OK) return rc;
  const cas::ActLayout L = cas::act_layout(*cfg);
  if (act_bytes < L.total) return CAS_ENOMEM;
  if (!cas::aligned256(d_act)) return CAS_EINVAL;
  const int qd = cfg->n_q_heads * cfg->head_dim, kvd = cfg->n_kv_heads * cfg->head_dim;
  auto shape_ok = [](const cas_tensor& t, int64_t rows, int64_t cols) {
    return t.d_spec && t.d_verif && t.desc.rows == rows && t.desc.cols == cols;
  };
  for (int l = 0; l < cfg->n_layers; ++l) {
    const cas_layer_weights& lw = w->layers[l];
    if (!shape_ok(lw.wqkv, qd + 2 * kvd, cfg->hidden) || !shape_ok(lw.wo, cfg->hidden, qd) ||
        !shape_ok(lw.wgu, 2 * (int64_t)cfg->ffn, cfg->hidden) || !shape_ok(lw.wd, cfg->hidden, cfg->ffn) ||
        !lw.d_g_attn || !lw.d_g_ffn)
      return CAS_EINVAL;
  }
  if (!shape_ok(w->lm_head, cfg->vocab, cfg->hidden)) return CAS_EINVAL;
  cas_model* m = new (std::nothrow) cas_model();
  if (!m) return CAS_ENOMEM;
  m->cfg = *cfg;
  m->layers = new (std::nothrow) cas_layer_weights[cfg->n_layers];
  if (!m->layers) { delete m; return CAS_ENOMEM; }
  std::copy(w->layers, w->layers + cfg->n_layers, m->layers);
  m->lm_head = w->lm_head;
  m->unary.resize(4 * (size_t)cfg->n_layers + 1);
  m->d_embed = w->d_embed; m->d_g_final = w->d_g_final; m->d_rope = w->d_rope;
  char* b = (char*)d_act;
  m->h = (uint16_t*)(b + L.h); m->xn = (uint16_t*)(b + L.xn); m->q = (uint16_t*)(b + L.q);
  m->ao = (uint16_t*)(b + L.ao); m->act = (uint16_t*)(b + L.act);
  m->knew = (uint16_t*)(b + L.knew); m->vnew = (uint16_t*)(b + L.vnew);
  m->y = (float*)(b + L.y); m->logits = (float*)(b + L.logits);
  m->tok = (int32_t*)(b + L.tok); m->tgt = (int32_t*)(b + L.tgt);
  m->amax_v = (float*)(b + L.amax_v); m->amax_i = (int32_t*)(b + L.amax_i);
  *out = m;
  return CAS_OK;
}

// the tensor (layer, which) of the model and its alternative-form record; false if there is none
static bool model_tensor(cas_model* m, int layer, int which, const cas_tensor** T, cas_model::UnaryRef** U) {
  if (!m || layer < -1 || layer >= m->cfg.n_layers || (layer >= 0 && (which < 0 || which > 3))) return false;
  *T = &m->lm_head;
  if (layer >= 0) {
    cas_layer_weights& lw = m->layers[layer];
    *T = which == 0 ? &lw.wqkv : which == 1 ? &lw.wo : which == 2 ? &lw.wgu : &lw.wd;
  }
  *U = layer < 0 ? &m->unary.back() : &m->unary[4 * (size_t)layer + which];
  return true;
}

// another form must be the re-coding of this very tensor: same shape, kept count, truncation, stream widths
static bool same_matrix(const cas_wdesc& a, const cas_wdesc& b) {
  return a.rows == b.rows && a.cols == b.cols && a.K == b.K && a.t == b.t && a.bw == b.bw && a.sw == b.sw &&
         a.lw == b.lw && a.pw == b.pw;
}

int cas_model_use_unary(cas_model* m, int layer, int which, const cas_udesc* udesc, const void* d_uspec) {
  const cas_tensor* T;
  cas_model::UnaryRef* U;
  if (!model_tensor(m, layer, which, &T, &U)) return CAS_EINVAL;
  if (!udesc) { U->on = false; return CAS_OK; }
  if (!d_uspec || !cas::aligned256(d_uspec)) return CAS_EINVAL;
  // ... and the verification data stays the tensor's own
  if (!same_matrix(udesc->base, T->desc) || udesc->base.off_lo != T->desc.off_lo ||
      udesc->base.off_pruned != T->desc.off_pruned)
    return CAS_EINVAL;
  U->u = *udesc;
  U->d_uspec = d_uspec;
  U->on = true;
  U->mx_on = false;
  return CAS_OK;
}

int cas_model_use_mx(cas_model* m, int layer, int which, const cas_mxdesc* mx, const void* d_mxspec,
                     const void* d_mxverif) {
  const cas_tensor* T;
  cas_model::UnaryRef* U;
  if (!model_tensor(m, layer, which, &T, &U)) return CAS_EINVAL;
  if (!mx) { U->mx_on = false; return CAS_OK; }
  if (!d_mxspec || !d_mxverif || !cas::aligned256(d_mxspec) || !cas::aligned256(d_mxverif)) return CAS_EINVAL;
  if (!cas::mxdesc_ok(mx) || !same_matrix(mx->base, T->desc)) return CAS_EINVAL;
  U->mx = *mx;
  U->d_mxspec = d_mxspec;
  U->d_mxverif = d_mxverif;
  U->mx_on = true;
  U->on = false;
  return CAS_OK;
}

int cas_model_destroy(cas_model* m) {
  if (m) { delete[] m->layers; delete m; }
  return CAS_OK;
}

static int check_step(cas_ctx* ctx, cas_model* m, cas_kv* kv, int seq) {
  if (!ctx || !m || !kv || seq < 0 || seq >= kv->desc.max_seqs || seq >= cas::model_seqs(m->cfg)) return CAS_EINVAL;
  if (kv->desc.n_layers != m->cfg.n_layers || kv->desc.n_kv_heads != m->cfg.n_kv_heads) return CAS_EINVAL;
  return CAS_OK;
}

int cas_draft_step(cas_ctx* ctx, cas_model* m, cas_kv* kv, int seq, const int32_t* d_token_in, int slot,
                   int32_t* d_token_out, float* d_logits) {
  if (check_step(ctx, m, kv, seq) != CAS_OK || !d_token_in || !d_token_out || slot < 0) return CAS_EINVAL;
  const cas::ColGroup g{seq, 1, slot};
  return cas::forward(ctx, m, kv, &g, 1, d_token_in, false, d_token_out, d_logits);
}

int cas_verify_step(cas_ctx* ctx, cas_model* m, cas_kv* kv, int seq, const int32_t* d_tokens, int k,
                    int32_t* d_target, float* d_logits) {
  if (check_step(ctx, m, kv, seq) != CAS_OK || !d_tokens || k < 0) return CAS_EINVAL;
  const cas::ColGroup g{seq, k + 1, 0};
  return cas::forward(ctx, m, kv, &g, 1, d_tokens, true, d_target, d_logits);
}

int cas_draft_step_multi(cas_ctx* ctx, cas_model* m, cas_kv* kv, int n_seqs, const int32_t* h_seqs,
                         const int32_t* h_slots, const int32_t* d_tokens_in, int32_t* d_tokens_out) {
  if (!ctx || !m || !kv || n_seqs < 1 || n_seqs > 4 || !h_seqs || !h_slots || !d_tokens_in || !d_tokens_out)
    return CAS_EINVAL;
  if (kv->desc.n_layers != m->cfg.n_layers || kv->desc.n_kv_heads != m->cfg.n_kv_heads) return CAS_EINVAL;
  cas::ColGroup g[4];
  for (int i = 0; i < n_seqs; ++i) g[i] = cas::ColGroup{h_seqs[i], 1, h_slots[i]};
  return cas::forward(ctx, m, kv, g, n_seqs, d_tokens_in, false, d_tokens_out, nullptr);
}

// Verification columns of several sequences: sequences are taken in order, as many per pass as
// fit max_cols columns (a pass reads every weight once; a column's value does not depend on
// how the sequences are split over passes).
static int verify_groups(cas_ctx* ctx, cas_model* m, cas_kv* kv, int n_seqs, const int32_t* h_seqs, const int32_t* h_k,
                         const int32_t* d_tokens, int32_t* d_target) {
  cas::ColGroup g[16];
  for (int s = 0, off = 0; s < n_seqs;) {
    int ng = 0, cols = 0;
    while (s + ng < n_seqs && ng < 16 && cols + h_k[s + ng] + 1 <= m->cfg.max_cols) {
      g[ng] = cas::ColGroup{h_seqs[s + ng], h_k[s + ng] + 1, 0};
      cols += h_k[s + ng] + 1;
      ++ng;
    }
    if (ng == 0) return CAS_EINVAL;  // one sequence alone exceeds max_cols
    int rc = cas::forward(ctx, m, kv, g, ng, d_tokens + off, true, d_target + off, nullptr);
    if (rc != CAS_OK) return rc;
    s += ng;
    off += cols;
  }
  return CAS_OK;
}

int cas_verify_step_multi(cas_ctx* ctx, cas_model* m, cas_kv* kv, int n_seqs, const int32_t* h_seqs,
                          const int32_t* h_k, const int32_t* d_tokens, int32_t* d_target) {
  if (!ctx || !m || !kv || n_seqs < 1 || n_seqs > 16 || !h_seqs || !h_k || !d_tokens || !d_target) return CAS_EINVAL;
  if (kv->desc.n_layers != m->cfg.n_layers || kv->desc.n_kv_heads != m->cfg.n_kv_heads) return CAS_EINVAL;
  for (int i = 0; i < n_seqs; ++i)
    if (h_k[i] < 0) return CAS_EINVAL;
  return verify_groups(ctx, m, kv, n_seqs, h_seqs, h_k, d_tokens, d_target);
}

int cas_commit(cas_ctx* ctx, cas_model* m, cas_kv* kv, int seq, int n_accepted) {
  if (check_step(ctx, m, kv, seq) != CAS_OK || n_accepted < 0 || n_accepted + 1 > m->cfg.max_cols) return CAS_EINVAL;
  const cas_model_cfg& c = m->cfg;
  const int kvd = c.n_kv_heads * c.head_dim, n = n_accepted + 1;
  const int64_t cap = (int64_t)kv->desc.max_pages_per_seq * kv->desc.page_tokens;
  if ((int64_t)kv->h_len[seq] + n > cap) return CAS_ENOMEM;
  // all layers in one launch: the slots of a sequence are [layer][max_cols][kv heads * 128]
  const size_t slots = (size_t)seq * c.n_layers * c.max_cols * kvd;
  int rc = cas::launch_kv_append_layers(ctx, kv, 0, c.n_layers, (size_t)c.max_cols * kvd, seq, m->knew + slots,
                                        m->vnew + slots, n, kv->h_len[seq]);
  if (rc != CAS_OK) return rc;
  kv->h_len[seq] += n;
  return CAS_OK;
}

int cas_spec_round(cas_ctx* ctx, cas_model* m, cas_kv* kv, int seq, int32_t pending, int k, int32_t* h_out,
                   int32_t* n_accepted) {
  if (check_step(ctx, m, kv, seq) != CAS_OK || !h_out || !n_accepted || k < 0 || k + 1 > m->cfg.max_cols)
    return CAS_EINVAL;
  CAS_HIP(ctx, hipMemcpyAsync(m->tok, &pending, sizeof(int32_t), hipMemcpyHostToDevice, ctx->stream));
  for (int i = 0; i < k; ++i) {
    const cas::ColGroup g{seq, 1, i};
    int rc = cas::forward(ctx, m, kv, &g, 1, m->tok + i, false, m->tok + i + 1, nullptr);
    if (rc != CAS_OK) return rc;
  }
  const cas::ColGroup gv{seq, k + 1, 0};
  int rc = cas::forward(ctx, m, kv, &gv, 1, m->tok, true, m->tgt, nullptr);
  if (rc != CAS_OK) return rc;
  int32_t h_tok[17], h_tgt[17];
  CAS_HIP(ctx, hipMemcpyAsync(h_tok, m->tok, sizeof(int32_t) * (k + 1), hipMemcpyDeviceToHost, ctx->stream));
  CAS_HIP(ctx, hipMemcpyAsync(h_tgt, m->tgt, sizeof(int32_t) * (k + 1), hipMemcpyDeviceToHost, ctx->stream));
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  rc = cas_accept(h_tok + 1, h_tgt, k, n_accepted, h_out);
  if (rc != CAS_OK) return rc;
  return cas_commit(ctx, m, kv, seq, *n_accepted);
}

int cas_spec_round_multi(cas_ctx* ctx, cas_model* m, cas_kv* kv, int n_seqs, const int32_t* h_seqs,
                         const int32_t* h_pending, int k, int32_t* h_out, int32_t* h_n_accepted) {
  if (!ctx || !m || !kv || n_seqs < 1 || n_seqs > 4 || !h_seqs || !h_pending || !h_out || !h_n_accepted || k < 0)
    return CAS_EINVAL;
  const int steps = k + 1, total = steps * n_seqs;
  if (steps > m->cfg.max_cols) return CAS_EINVAL;
  if (kv->desc.n_layers != m->cfg.n_layers || kv->desc.n_kv_heads != m->cfg.n_kv_heads) return CAS_EINVAL;
  int32_t* step_major = m->tok;                      // [steps][n_seqs]
  int32_t* seq_major = m->tok + 4 * m->cfg.max_cols;   // [n_seqs][steps]
  CAS_HIP(ctx, hipMemcpyAsync(step_major, h_pending, sizeof(int32_t) * n_seqs, hipMemcpyHostToDevice, ctx->stream));
  cas::ColGroup g[4];
  for (int i = 0; i < k; ++i) {
    for (int s = 0; s < n_seqs; ++s) g[s] = cas::ColGroup{h_seqs[s], 1, i};
    int rc = cas::forward(ctx, m, kv, g, n_seqs, step_major + i * n_seqs, false, step_major + (i + 1) * n_seqs, nullptr);
    if (rc != CAS_OK) return rc;
  }
  hipLaunchKernelGGL(cas::transpose_tokens_kernel, dim3(1), dim3(64), 0, ctx->stream, step_major, seq_major, steps,
                     n_seqs);  // total <= 4 * 16 = 64 threads
  int32_t h_k[4];
  for (int s = 0; s < n_seqs; ++s) h_k[s] = k;
  int rc = verify_groups(ctx, m, kv, n_seqs, h_seqs, h_k, seq_major, m->tgt);
  if (rc != CAS_OK) return rc;
  int32_t h_tok[64], h_tgt[64];
  CAS_HIP(ctx, hipMemcpyAsync(h_tok, seq_major, sizeof(int32_t) * total, hipMemcpyDeviceToHost, ctx->stream));
  CAS_HIP(ctx, hipMemcpyAsync(h_tgt, m->tgt, sizeof(int32_t) * total, hipMemcpyDeviceToHost, ctx->stream));
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  for (int s = 0; s < n_seqs; ++s) {
    rc = cas_accept(h_tok + s * steps + 1, h_tgt + s * steps, k, h_n_accepted + s, h_out + s * steps);
    if (rc != CAS_OK) return rc;
    rc = cas_commit(ctx, m, kv, h_seqs[s], h_n_accepted[s]);
    if (rc != CAS_OK) return rc;
  }
  return CAS_OK;
}

int cas_token_probs(cas_ctx* ctx, const float* d_logits, int vocab, int n, const int32_t* d_tokens, float* d_probs) {
  if (!ctx || n < 0 || vocab < 1 || (n > 0 && (!d_logits || !d_tokens || !d_probs))) return CAS_EINVAL;
  if (n == 0) return CAS_OK;
  hipLaunchKernelGGL(cas::token_prob_kernel, dim3(n), dim3(cas::kProbThreads), 0, ctx->stream, d_logits, vocab, d_tokens,
                     d_probs);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

size_t cas_spec_round_sampling_scratch_floats(int vocab, int k) {
  return (vocab < 1 || k < 0) ? 0 : (size_t)(2 * k + 1) * (size_t)vocab + 2 * (size_t)k;
}

int cas_spec_round_sampling(cas_ctx* ctx, cas_model* m, cas_kv* kv, int seq, int32_t pending, int k, const double* h_r,
                            float* d_scratch, int32_t* h_out, int32_t* n_accepted, double* h_p, double* h_q) {
  if (check_step(ctx, m, kv, seq) != CAS_OK || !h_out || !n_accepted || k < 0 || k + 1 > m->cfg.max_cols || k > 16)
    return CAS_EINVAL;
  if (k > 0 && (!h_r || !d_scratch)) return CAS_EINVAL;
  const size_t vocab = (size_t)m->cfg.vocab;
  float* dlog = d_scratch;                     // [k][vocab] logits of the draft passes
  float* vlog = d_scratch + (size_t)k * vocab; // [k+1][vocab] logits of the verification pass
  float* dq = vlog + (size_t)(k + 1) * vocab;  // [k] draft probabilities, then [k] target probabilities
  float* dp = dq + k;
  CAS_HIP(ctx, hipMemcpyAsync(m->tok, &pending, sizeof(int32_t), hipMemcpyHostToDevice, ctx->stream));
  for (int i = 0; i < k; ++i) {
    const cas::ColGroup g{seq, 1, i};
    int rc = cas::forward(ctx, m, kv, &g, 1, m->tok + i, false, m->tok + i + 1, dlog + (size_t)i * vocab);
    if (rc != CAS_OK) return rc;
  }
  const cas::ColGroup gv{seq, k + 1, 0};
  int rc = cas::forward(ctx, m, kv, &gv, 1, m->tok, true, m->tgt, k > 0 ? vlog : nullptr);
  if (rc != CAS_OK) return rc;
  // q_i: draft pass i's softmax at the token it drafted; p_i: the target's softmax after the
  // same prefix (verification column i - 1) at that token
  rc = cas_token_probs(ctx, dlog, (int)vocab, k, m->tok + 1, dq);
  if (rc != CAS_OK) return rc;
  rc = cas_token_probs(ctx, vlog, (int)vocab, k, m->tok + 1, dp);
  if (rc != CAS_OK) return rc;
  int32_t h_tok[17], h_tgt[17];
  float h_pq[32];
  CAS_HIP(ctx, hipMemcpyAsync(h_tok, m->tok, sizeof(int32_t) * (k + 1), hipMemcpyDeviceToHost, ctx->stream));
  CAS_HIP(ctx, hipMemcpyAsync(h_tgt, m->tgt, sizeof(int32_t) * (k + 1), hipMemcpyDeviceToHost, ctx->stream));
  if (k > 0) CAS_HIP(ctx, hipMemcpyAsync(h_pq, dq, sizeof(float) * 2 * k, hipMemcpyDeviceToHost, ctx->stream));
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  double p[16], q[16];
  for (int i = 0; i < k; ++i) {
    q[i] = (double)h_pq[i];
    p[i] = (double)h_pq[k + i];
    if (h_q) h_q[i] = q[i];
    if (h_p) h_p[i] = p[i];
  }
  rc = cas_accept_sampling(p, q, h_r, k, n_accepted);
  if (rc != CAS_OK) return rc;
  for (int i = 0; i < *n_accepted; ++i) h_out[i] = h_tok[i + 1];
  h_out[*n_accepted] = h_tgt[*n_accepted];
  return cas_commit(ctx, m, kv, seq, *n_accepted);
}

int cas_dense_decode_step(cas_ctx* ctx, cas_model* m, const cas_dense_layer* h_layers, const uint16_t* d_lm_head,
                          uint16_t* d_kcache, uint16_t* d_vcache, int len, const int32_t* d_token_in,
                          int32_t* d_token_out, float* d_logits) {
  if (!ctx || !m || !h_layers || !d_lm_head || !d_kcache || !d_vcache || !d_token_in || len < 0) return CAS_EINVAL;
  const cas_model_cfg& c = m->cfg;
  if (len + 1 > c.max_pos) return CAS_EINVAL;
  const int qd = c.n_q_heads * c.head_dim, kvd = c.n_kv_heads * c.head_dim;
  hipStream_t st = ctx->stream;
  float* logits = d_logits ? d_logits : m->logits;
  hipLaunchKernelGGL(cas::embed_kernel, dim3(1), dim3(256), 0, st, d_token_in, m->d_embed, m->h, c.hidden, c.vocab);
  for (int l = 0; l < c.n_layers; ++l) {
    const cas_dense_layer& D = h_layers[l];
    const cas_layer_weights& L = m->layers[l];
    if (!D.d_wqkv || !D.d_wo || !D.d_wgu || !D.d_wd) return CAS_EINVAL;
    uint16_t* kc = d_kcache + (size_t)l * c.max_pos * kvd;
    uint16_t* vc = d_vcache + (size_t)l * c.max_pos * kvd;
    hipLaunchKernelGGL(cas::rmsnorm_kernel, dim3(1), dim3(cas::kNormThreads), 0, st, m->h, L.d_g_attn, m->xn, c.hidden,
                       c.rms_eps);
    CAS_TRY(cas_gemv_bf16(ctx, D.d_wqkv, qd + 2 * kvd, c.hidden, c.hidden, m->xn, m->y));
    CAS_TRY(cas::launch_attention_dense(ctx, c.n_kv_heads, c.n_q_heads, kc, vc, len, m->y, qd + 2 * kvd, m->d_rope, m->ao));
    CAS_TRY(cas_gemv_bf16(ctx, D.d_wo, c.hidden, qd, qd, m->ao, m->y));
    hipLaunchKernelGGL(cas::residual_add_kernel, dim3((c.hidden + 255) / 256), dim3(256), 0, st, m->h, m->y, c.hidden);
    hipLaunchKernelGGL(cas::rmsnorm_kernel, dim3(1), dim3(cas::kNormThreads), 0, st, m->h, L.d_g_ffn, m->xn, c.hidden,
                       c.rms_eps);
    CAS_TRY(cas_gemv_bf16(ctx, D.d_wgu, 2 * (int64_t)c.ffn, c.hidden, c.hidden, m->xn, m->y));
    hipLaunchKernelGGL(cas::swiglu_kernel, dim3((c.ffn + 255) / 256), dim3(256), 0, st, m->y, m->act, c.ffn);
    CAS_TRY(cas_gemv_bf16(ctx, D.d_wd, c.hidden, c.ffn, c.ffn, m->act, m->y));
    hipLaunchKernelGGL(cas::residual_add_kernel, dim3((c.hidden + 255) / 256), dim3(256), 0, st, m->h, m->y, c.hidden);
  }
  hipLaunchKernelGGL(cas::rmsnorm_kernel, dim3(1), dim3(cas::kNormThreads), 0, st, m->h, m->d_g_final, m->xn, c.hidden,
                     c.rms_eps);
  CAS_TRY(cas_gemv_bf16(ctx, d_lm_head, c.vocab, c.hidden, c.hidden, m->xn, logits));
  if (d_token_out) {
    hipLaunchKernelGGL(cas::argmax_part_kernel, dim3(cas::kArgmaxSlices, 1), dim3(256), 0, st, logits, c.vocab, m->amax_v,
                       m->amax_i);
    hipLaunchKernelGGL(cas::argmax_final_kernel, dim3(1), dim3(64), 0, st, m->amax_v, m->amax_i, d_token_out);
  }
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

int cas_prefill(cas_ctx* ctx, cas_model* m, cas_kv* kv, int seq, const int32_t* d_tokens, int n) {
  if (check_step(ctx, m, kv, seq) != CAS_OK || !d_tokens || n < 0) return CAS_EINVAL;
  for (int done = 0; done < n;) {
    const int nc = std::min(n - done, cas::seq_cols_max(m->cfg));
    const cas::ColGroup g{seq, nc, 0};
    int rc = cas::forward(ctx, m, kv, &g, 1, d_tokens + done, true, nullptr, nullptr);
    if (rc != CAS_OK) return rc;
    rc = cas_commit(ctx, m, kv, seq, nc - 1);
    if (rc != CAS_OK) return rc;
    done += nc;
  }
  return CAS_OK;
}

}  // extern "C"
