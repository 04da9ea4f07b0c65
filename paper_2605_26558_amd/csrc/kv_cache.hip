// Compressed, paged KV cache: online formatting of new K/V vectors (Sec. 5.1 encoder,
// Sec. 4.2 per-token magnitude pruning) and a reference read-back.
//
// A tile holds the vectors of one (layer, page, K-or-V, kv head): page_tokens rows of
// head_dim = 128 values, K kept per row, in the same four-stream layout as a weight matrix
// (bitmap and spec in the speculation pool; lo and pruned in the verification pool).
#include "cas_device.hpp"
#include "cas_internal.hpp"

namespace cas {

// One wave formats one 128-value vector.  Keys (magnitude << 7 | 127 - column) are unique, so
// the K-th largest key is found bit by bit with wave ballots and "key >= threshold" keeps
// exactly K values with ties going to the lower column.
__global__ __launch_bounds__(64) void kv_append_kernel(KvGeom g, uint32_t* spec_pool, uint32_t* verif_pool,
                                                       const int32_t* __restrict__ page_row, int layer0, int pos0,
                                                       const uint16_t* __restrict__ Kn,
                                                       const uint16_t* __restrict__ Vn, size_t layer_stride) {
  __shared__ uint32_t stage[3 * 64 + 8];  // sw + lw + pw <= 16*128/32 = 64 words (+ rounding)
  const int lane = threadIdx.x;
  // grid.z = 2 * (layers of this launch): the vectors of layer layer0 + i start i * layer_stride
  // values after those of layer0
  const int tok = blockIdx.x, head = blockIdx.y, kv = blockIdx.z & 1, layer = layer0 + (blockIdx.z >> 1);
  const uint16_t* src = (kv ? Vn : Kn) + (size_t)(blockIdx.z >> 1) * layer_stride +
                        ((size_t)tok * g.n_kv_heads + head) * 128;
  const uint32_t v0 = src[lane], v1 = src[lane + 64];
  const uint32_t key0 = ((v0 & 0x7FFFu) << 7) | (uint32_t)(127 - lane);
  const uint32_t key1 = ((v1 & 0x7FFFu) << 7) | (uint32_t)(63 - lane);
  uint32_t T = 0;
  bool k0 = false, k1 = false;
  if (g.K > 0) {
    for (int bit = 21; bit >= 0; --bit) {
      uint32_t cand = T | (1u << bit);
      int cnt = __popcll(__builtin_amdgcn_ballot_w64(key0 >= cand)) + __popcll(__builtin_amdgcn_ballot_w64(key1 >= cand));
      if (cnt >= g.K) T = cand;
    }
    k0 = key0 >= T;
    k1 = key1 >= T;
  }
  const uint64_t m01 = __builtin_amdgcn_ballot_w64(k0), m23 = __builtin_amdgcn_ballot_w64(k1);
  const uint32_t below = (uint32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(m01 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m01, 0u));
  const uint32_t below2 = (uint32_t)__builtin_amdgcn_mbcnt_hi((uint32_t)(m23 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m23, 0u));
  const uint32_t r0 = below, r1 = (uint32_t)__popcll(m01) + below2;

  for (int i = lane; i < g.sw + g.lw + g.pw; i += 64) stage[i] = 0;
  __syncthreads();
  uint32_t* st_spec = stage;
  uint32_t* st_lo = stage + g.sw;
  uint32_t* st_pr = st_lo + g.lw;
  const int fw = g.mx ? 9 - g.t : 16 - g.t;
  const uint32_t lomask = (1u << g.t) - 1u;
  // shared-exponent form: the exponent of a 32-channel block is the largest among its kept values
  // (0 for a block without any); lanes 0..31 / 32..63 hold blocks 0 / 1 in v0 and blocks 2 / 3 in v1
  int E0 = 0, E1 = 0;
  if (g.mx) {
    E0 = k0 ? eff_exponent(v0) : 0;
    E1 = k1 ? eff_exponent(v1) : 0;
#pragma unroll
    for (int d = 1; d < 32; d <<= 1) {
      E0 = max(E0, __shfl_xor(E0, d));
      E1 = max(E1, __shfl_xor(E1, d));
    }
  }
  auto put = [&](uint32_t* s, uint32_t bit, uint32_t v, int width) {
    uint32_t w = bit >> 5, sh = bit & 31;
    atomicOr(&s[w], v << sh);
    if (sh + width > 32) atomicOr(&s[w + 1], v >> (32 - sh));
  };
  auto emit = [&](bool kept, uint32_t v, uint32_t rank, uint32_t col, int E) {
    if (kept) {
      if (g.mx) {  // sign + magnitude: the significand shifted down to the block's exponent
        const int sh = E - eff_exponent(v);
        const uint32_t mag = sh < 8 ? significand(v) >> sh : 0u;
        put(st_spec, rank * fw, ((v >> 15) << (8 - g.t)) | (mag >> g.t), fw);
        if (g.t) put(st_lo, rank * g.t, mag & lomask, g.t);
      } else {
        put(st_spec, rank * fw, v >> g.t, fw);
        if (g.t) put(st_lo, rank * g.t, v & lomask, g.t);
      }
    } else {
      put(st_pr, (col - rank) * 16, v, 16);
    }
  };
  emit(k0, v0, r0, (uint32_t)lane, E0);
  emit(k1, v1, r1, (uint32_t)lane + 64u, E1);
  __syncthreads();

  const int pos = pos0 + tok;
  const int page = page_row[pos / g.page_tokens];
  if (page < 0 || page >= g.n_pages) return;  // a page table entry outside the pool: nothing is written
  const int row = pos % g.page_tokens;
  const size_t tile = (((size_t)layer * g.n_pages + page) * 2 + kv) * g.n_kv_heads + head;
  uint32_t* ts = spec_pool + tile * g.tile_spec_words;
  uint32_t* tv = verif_pool + tile * g.tile_verif_words;
  if (lane < 4) {
    uint64_t m = lane < 2 ? m01 : m23;
    ts[row * 4 + lane] = (uint32_t)(m >> ((lane & 1) * 32));
  }
  if (g.mx) {  // the four block exponents of the vector, block j in byte j
    const int e01 = __shfl(E0, 0) | (__shfl(E0, 32) << 8), e23 = __shfl(E1, 0) | (__shfl(E1, 32) << 8);
    if (lane == 0) ts[g.page_tokens * 4 + row] = (uint32_t)(e01 | (e23 << 16));
  }
  uint32_t* dspec = ts + g.spec_off + row * g.sw;
  uint32_t* dlo = tv + row * g.lw;
  uint32_t* dpr = tv + g.page_tokens * g.lw + row * g.pw;
  for (int i = lane; i < g.sw; i += 64) dspec[i] = st_spec[i];
  for (int i = lane; i < g.lw; i += 64) dlo[i] = st_lo[i];
  for (int i = lane; i < g.pw; i += 64) dpr[i] = st_pr[i];
}

// Reference read-back of cached vectors to dense bf16 (full == 0: zero-padded draft view).
__global__ __launch_bounds__(128) void kv_read_kernel(KvGeom g, const uint32_t* spec_pool, const uint32_t* verif_pool,
                                                      const int32_t* __restrict__ page_row, int layer, int pos0,
                                                      int full, uint16_t* Ko, uint16_t* Vo) {
  const int col = threadIdx.x;
  const int tok = blockIdx.x, head = blockIdx.y, kv = blockIdx.z;
  const int pos = pos0 + tok;
  int page = page_row[pos / g.page_tokens];
  if (page < 0 || page >= g.n_pages) {  // a page table entry outside the pool reads as zeros
    (kv ? Vo : Ko)[((size_t)tok * g.n_kv_heads + head) * 128 + col] = 0;
    return;
  }
  const int row = pos % g.page_tokens;
  const size_t tile = (((size_t)layer * g.n_pages + page) * 2 + kv) * g.n_kv_heads + head;
  const uint32_t* ts = spec_pool + tile * g.tile_spec_words;
  const uint32_t* tv = verif_pool + tile * g.tile_verif_words;
  const uint32_t* bm = ts + row * 4;
  const int j = col >> 5, c = col & 31;
  uint32_t p = 0;
  for (int i = 0; i < j; ++i) p += __popc(bm[i]);
  const uint32_t m = bm[j];
  p += __popc(m & ((1u << c) - 1u));
  const int fw = g.mx ? 9 - g.t : 16 - g.t;
  uint32_t v;
  if ((m >> c) & 1u) {
    v = read_field(ts + g.spec_off + row * g.sw, p * fw, fw);
    const uint32_t lo = (full && g.t) ? read_field(tv + row * g.lw, p * g.t, g.t) : 0u;
    if (g.mx) {
      const int E = (int)((ts[g.page_tokens * 4 + row] >> (8 * j)) & 0xFFu);
      v = mx_word(v >> (8 - g.t), E, ((v & ((1u << (8 - g.t)) - 1u)) << g.t) | lo);
    } else {
      v = (v << g.t) | lo;
    }
  } else {
    v = full ? read_field(tv + g.page_tokens * g.lw + row * g.pw, ((uint32_t)col - p) * 16, 16) : 0u;
  }
  uint16_t* dst = (kv ? Vo : Ko) + ((size_t)tok * g.n_kv_heads + head) * 128;
  dst[col] = (uint16_t)v;
}

int launch_kv_append(cas_ctx* ctx, cas_kv* kv, int layer, int seq, const uint16_t* K, const uint16_t* V, int n_tok,
                     int pos0) {
  return launch_kv_append_layers(ctx, kv, layer, 1, 0, seq, K, V, n_tok, pos0);
}

int launch_kv_append_layers(cas_ctx* ctx, cas_kv* kv, int layer0, int n_layers, size_t layer_stride, int seq,
                            const uint16_t* K, const uint16_t* V, int n_tok, int pos0) {
  if (n_tok <= 0 || n_layers <= 0) return CAS_OK;
  const KvGeom& g = kv->geom;
  dim3 grid(n_tok, g.n_kv_heads, 2 * n_layers);
  hipLaunchKernelGGL(kv_append_kernel, grid, dim3(64), 0, ctx->stream, g, (uint32_t*)kv->d_spec,
                     (uint32_t*)kv->d_verif, kv->d_page_table + (size_t)seq * g.max_pages_per_seq, layer0, pos0, K, V,
                     layer_stride);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

int launch_kv_read(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int pos0, int n_tok, int full, uint16_t* K,
                   uint16_t* V) {
  if (n_tok <= 0) return CAS_OK;
  const KvGeom& g = kv->geom;
  dim3 grid(n_tok, g.n_kv_heads, 2);
  hipLaunchKernelGGL(kv_read_kernel, grid, dim3(128), 0, ctx->stream, g, (const uint32_t*)kv->d_spec,
                     (const uint32_t*)kv->d_verif, kv->d_page_table + (size_t)seq * g.max_pages_per_seq, layer, pos0,
                     full, K, V);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

}  // namespace cas
