// Host-side internals of the library: context, error plumbing, kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/cassandra.h"

#include <atomic>
#include <vector>

namespace cas {
enum ProfClass { PROF_GEMV_DRAFT = 0, PROF_GEMM_VERIFY = 1, PROF_ATTN_DRAFT = 2, PROF_ATTN_VERIFY = 3, PROF_NCLASS = 4 };
struct ProfRec { int cls; double bytes; hipEvent_t e0, e1; };
}  // namespace cas

struct cas_ctx {
  bool prof_on = false;
  std::vector<cas::ProfRec> prof;
  hipStream_t stream;
  void* d_ws;
  size_t ws_bytes;
  int last_hip;
  int num_cu;
  int lds_max;  // bytes of LDS one workgroup may use
  int device;   // the device that was current when the context was made
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
// geometry of the compressed KV cache as the kernels see it (sizes in 32-bit words)
struct KvGeom {
  int n_layers, n_kv_heads, page_tokens, n_pages, max_pages_per_seq;
  int K, t, sw, lw, pw;
  int tile_spec_words, tile_verif_words;
  // Shared-exponent form of the cache (mx != 0): a tile's speculation part is bitmap [64][4] |
  // one word per token with the exponents of its four 32-channel blocks | fields of 9-t bits
  // (sw words per token); spec_off = words in front of the field stream (256 raw, 320 shared).
  int mx, spec_off;
};
}  // namespace cas

struct cas_kv {
  cas_kv_desc desc;
  cas::KvGeom geom;
  void* d_spec;
  void* d_verif;
  const int32_t* d_page_table;
  int32_t* h_len;  // committed length of every sequence (host mirror; kernels get it as an argument)
};

namespace cas {
// Kernels that ask for more than 48 KB of dynamic LDS must be allowed to, once per device and
// kernel; one LdsLimit (a function-local static at the launch site) remembers what has been
// granted.  Two threads racing here both make the call, which is harmless.
struct LdsLimit {
  std::atomic<size_t> granted[16];
};
inline int allow_lds(cas_ctx* ctx, const void* kernel, size_t lds, LdsLimit& lim) {
  if (lds <= 48 * 1024) return CAS_OK;
  std::atomic<size_t>& g = lim.granted[ctx->device & 15];
  if (lds > g.load(std::memory_order_relaxed)) {
    CAS_HIP(ctx, hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    g.store(lds, std::memory_order_relaxed);
  }
  return CAS_OK;
}

inline bool aligned256(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255u) == 0; }

int launch_encode_weight(cas_ctx*, const uint16_t* W, int64_t ld, const float* act, const cas_wdesc&, void* spec, void* verif);
int launch_decode_weight(cas_ctx*, const cas_wdesc&, const void* spec, const void* verif, uint16_t* out, int64_t ld);
int launch_gemv_draft(cas_ctx*, const cas_wdesc&, const void* spec, const uint16_t* x, int batch, float* y);
int launch_gemv_draft_fused(cas_ctx*, const cas_wdesc&, const void* spec, const uint16_t* x, int batch, float* y,
                            const uint16_t* gain, float eps, int epi, uint16_t* out16);
int launch_gemm_verify(cas_ctx*, const cas_wdesc&, const void* spec, const void* verif, const uint16_t* X, int ncols, float* Y);
int launch_gemm_verify_fused(cas_ctx*, const cas_wdesc&, const void* spec, const void* verif, const uint16_t* X,
                             int ncols, float* Y, int epi, uint16_t* out16);
// unary.hip: rows [row0, row0 + nrows) of the raw spec stream (sw words per row) rebuilt from the unary form
int launch_unary_expand(cas_ctx*, const cas_udesc&, const void* uspec, int64_t row0, int nrows, uint32_t* out);
int launch_gemm_verify_unary_fused(cas_ctx*, const cas_udesc&, const void* uspec, const void* verif, const uint16_t* X,
                                   int ncols, float* Y, int epi, uint16_t* out16);
// mx.hip / gemm_verify_mx.hip
int launch_gemv_draft_mx_fused(cas_ctx*, const cas_mxdesc&, const void* mxspec, const uint16_t* x, float* y,
                               const uint16_t* gain, float eps, int epi, uint16_t* out16);
int launch_gemm_verify_mx_fused(cas_ctx*, const cas_mxdesc&, const void* mxspec, const void* mxverif, const uint16_t* X,
                                int ncols, float* Y, int epi, uint16_t* out16);
bool mxdesc_ok(const cas_mxdesc*);
int launch_kv_append(cas_ctx*, cas_kv*, int layer, int seq, const uint16_t* K, const uint16_t* V, int n_tok, int pos0);
// the same for n_layers consecutive layers in one launch; the vectors of layer layer0 + i start
// i * layer_stride values after K / V
int launch_kv_append_layers(cas_ctx*, cas_kv*, int layer0, int n_layers, size_t layer_stride, int seq,
                            const uint16_t* K, const uint16_t* V, int n_tok, int pos0);
int launch_kv_read(cas_ctx*, cas_kv*, int layer, int seq, int pos0, int n_tok, int full, uint16_t* K, uint16_t* V);
struct AttnCall {
  int layer, seq, full;        // full: 0 = speculation data only (draft), 1 = exact reconstruction
  const uint16_t* Q;           // [ncols][n_q_heads][128]
  int ncols, n_q_heads;
  const uint16_t* Knew;        // [n_new][n_kv_heads][128] uncompressed in-flight vectors
  const uint16_t* Vnew;
  int n_new;
  uint16_t* O;                 // [ncols][n_q_heads][128]
  // model path: split of the fp32 qkv projection fused in (see attention.hip); null otherwise
  const float* qkv = nullptr;
  int ystride = 0, slot0 = 0;
  const float* rope = nullptr;
  uint16_t* Kslot = nullptr;
  uint16_t* Vslot = nullptr;
};
int launch_attention(cas_ctx*, cas_kv*, const AttnCall&);
// the same with the partial results in the library's own fixed device array (no workspace, no
// allocation of any kind); CAS_ENOMEM beyond attention_static_capacity() bytes of partials
int launch_attention_static(cas_ctx*, cas_kv*, const AttnCall&);
size_t attention_static_capacity();
// the same for the sequences of one pass (same layer and form), four of them per pair of launches
int launch_attention_batch(cas_ctx*, cas_kv*, const AttnCall* calls, int n);
// plain bf16 attention of one decode step over an uncompressed cache (baseline for context figures)
int launch_attention_dense(cas_ctx*, int n_kv_heads, int n_q_heads, uint16_t* Kc, uint16_t* Vc, int len,
                           const float* qkv, int ystride, const float* rope, uint16_t* O);
// Brackets one kernel launch with HIP events on the context stream when profiling is on.
struct ProfScope {
  cas_ctx* ctx;
  bool on;
  ProfRec rec;
  ProfScope(cas_ctx* c, int cls, double bytes) : ctx(c), on(c && c->prof_on) {
    if (!on) return;
    rec.cls = cls; rec.bytes = bytes;
    if (hipEventCreate(&rec.e0) != hipSuccess || hipEventCreate(&rec.e1) != hipSuccess) { on = false; return; }
    (void)hipEventRecord(rec.e0, ctx->stream);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(rec.e1, ctx->stream);
    ctx->prof.push_back(rec);
  }
};
}  // namespace cas
