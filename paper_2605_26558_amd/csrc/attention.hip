// Attention of the decode step over the compressed, paged KV cache (Fig. 2_1 structure;
// Sec. 4.1 decides which data a pass may read): the draft pass rebuilds K and V from the
// speculation data with zero padding, the verification pass rebuilds them exactly from both
// pools.  The vectors of the in-flight tokens (draft tokens not yet verified, or the k+1
// columns of the verification pass) arrive uncompressed and are placed at the page rows their
// positions will occupy, and a split always covers the same fixed number of pages: the value
// of a query therefore depends only on the tokens it sees, not on whether they are already
// committed, nor on the number of columns or the total length.
//
// One workgroup handles one kv head and one page (64 positions) of the sequence:
//   1. thread (token r, word j) decodes its 32 channels of K into a 64 x 128 bf16 tile in LDS;
//   2. each wave multiplies its 16 tokens with the query rows (grouped-query: the query heads
//      of the group x columns share the kv head) by 16x16x16 bf16 MFMA; the scaled, masked
//      scores stay in the MFMA result registers;
//   3. softmax numerators of the page per query row: the row maximum and sum go through DPP
//      rotations inside a wave and a few LDS words across the four waves (kept for the
//      merge); probabilities are split into a bf16 head and a bf16 remainder, so the second
//      product keeps 16 mantissa bits, and stored over the query tile, which is dead by then;
//   4. the V tile is decoded transposed over the dead K tile and P V is formed in fp32 MFMA
//      registers.
// Partial (max, sum, output) of every page go to the workspace; a merge kernel combines them
// in a fixed order.
#include <algorithm>
#include <atomic>
#include "attention_kernel.inl"

namespace cas {

// the draft form (speculation data only) is compiled in attention_draft.hip
extern template int launch_mt<1, false, false>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<2, false, false>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<3, false, false>(cas_ctx*, const AttnBatch&, dim3);
// the forms over a cache with shared exponents: attention_mx.hip, attention_mx_draft.hip
extern template int launch_mt<1, true, true>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<2, true, true>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<3, true, true>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<4, true, true>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<5, true, true>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<1, false, true>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<2, false, true>(cas_ctx*, const AttnBatch&, dim3);
extern template int launch_mt<3, false, true>(cas_ctx*, const AttnBatch&, dim3);

// Combine the splits: o = sum_s e^{m_s - M} O_s / sum_s e^{m_s - M} l_s, rounded to bf16.
// One workgroup per (query row, kv head, half of the channels): the split weights are computed
// once into LDS, then thread (channel d, part p) sums the splits s = p, p + 8, ... with
// independent loads and the eight parts are added in part order (a fixed order: the result
// does not depend on timing, nor on how many rows ride along).
constexpr int kMergeParts = 8;
constexpr int kMergePre = 20;  // splits per thread whose outputs are requested before the weights exist
__global__ __launch_bounds__(512) void attn_merge_kernel(AttnBatch batch) {
  const AttnArgs a = attn_args_of(batch, blockIdx.z >> 1);  // blockIdx.z = 2 * sequence + channel half
  extern __shared__ float sw[];  // [nsplit] weights, then [kMergeParts][64] partial sums
  __shared__ float red[16];
  const int rr = blockIdx.x, head = blockIdx.y, tid = threadIdx.x;
  const int d = (blockIdx.z & 1) * 64 + (tid & 63), part = tid >> 6;
  const int R = a.ncols * a.grp;
  if (rr >= R) return;  // a sequence with fewer rows than the widest of the launch
  const size_t sstride = (size_t)a.g.n_kv_heads * R * kPartStride;
  const float* base = a.part + ((size_t)head * R + rr) * kPartStride;
  // everything this thread needs from the first 512 splits goes out in one batch: its split's
  // (max, sum) and the outputs of splits part, part + 8, ... of its channel
  float m0 = -INFINITY, l0 = 0.f;
  if (tid < a.nsplit) {
    m0 = base[tid * sstride + 128];
    l0 = base[tid * sstride + 129];
  }
  float o[kMergePre];
#pragma unroll
  for (int q = 0; q < kMergePre; ++q) {
    const int s = part + q * kMergeParts;
    o[q] = s < a.nsplit ? base[s * sstride + d] : 0.f;
  }
  float mx = m0;
  for (int s = tid + 512; s < a.nsplit; s += 512) mx = fmaxf(mx, base[s * sstride + 128]);
  mx = wave_max(mx);
  if ((tid & 63) == 0) red[tid >> 6] = mx;
  __syncthreads();
  float M = red[0];
#pragma unroll
  for (int w = 1; w < 8; ++w) M = fmaxf(M, red[w]);
  float den = 0.f;
  if (tid < a.nsplit) {
    const float w = (m0 == -INFINITY) ? 0.f : __expf(m0 - M);
    sw[tid] = w;
    den = w * l0;
  }
  for (int s = tid + 512; s < a.nsplit; s += 512) {
    float m = base[s * sstride + 128];
    float w = (m == -INFINITY) ? 0.f : __expf(m - M);
    sw[s] = w;
    den += w * base[s * sstride + 129];
  }
  den = wave_sum(den);
  if ((tid & 63) == 0) red[8 + (tid >> 6)] = den;
  __syncthreads();
  den = 0.f;
#pragma unroll
  for (int w = 0; w < 8; ++w) den += red[8 + w];
  float num = 0.f;
#pragma unroll
  for (int q = 0; q < kMergePre; ++q) {
    const int s = part + q * kMergeParts;
    if (s < a.nsplit) num += sw[s] * o[q];
  }
#pragma unroll 8
  for (int s = part + kMergePre * kMergeParts; s < a.nsplit; s += kMergeParts) num += sw[s] * base[s * sstride + d];
  float* ps = sw + a.nsplit;
  ps[part * 64 + (tid & 63)] = num;
  __syncthreads();
  if (part == 0) {
    num = ps[tid];
#pragma unroll
    for (int q = 1; q < kMergeParts; ++q) num += ps[q * 64 + tid];
    const int c = rr / a.grp, gi = rr - c * a.grp;
    a.O[((size_t)c * a.n_q_heads + head * a.grp + gi) * 128 + d] = f32_to_bf16(num / den);
  }
}

// Up to kAttnBatch sequences of one pass in one pair of launches (same layer, same form, same
// number of query heads); every sequence gets exactly what a launch of its own would give it.
// ws / ws_bytes: device memory for the per-split partial results; prof: bracket the launch with
// events when the context's measurement hooks are on (creates events: not for callers that may
// not allocate).
static int launch_attention_group(cas_ctx* ctx, cas_kv* kv, const AttnCall* calls, int n, void* ws, size_t ws_bytes,
                                  size_t* ws_used, bool prof) {
  const KvGeom& g = kv->geom;
  const AttnCall& c0 = calls[0];
  AttnBatch b{};
  AttnArgs& a = b.common;
  a.g = g;
  a.spec_pool = (const uint32_t*)kv->d_spec;
  a.verif_pool = (const uint32_t*)kv->d_verif;
  a.layer = c0.layer;
  a.n_q_heads = c0.n_q_heads; a.grp = c0.n_q_heads / g.n_kv_heads;
  a.ystride = c0.ystride; a.rope = c0.rope;
  a.scale = 0.08838834764831845f;  // 1 / sqrt(128)
  a.pages_per_split = kPagesPerSplit;  // fixed: a query's value must not depend on the length
  int max_r = 0, max_split = 0;
  double bytes = 0.0;
  for (int i = 0; i < n; ++i) {
    const AttnCall& c = calls[i];
    if (c.layer != c0.layer || c.full != c0.full || c.n_q_heads != c0.n_q_heads || c.ystride != c0.ystride ||
        c.rope != c0.rope || (c.qkv == nullptr) != (c0.qkv == nullptr))
      return CAS_EINVAL;
    AttnSeq& q = b.s[i];
    q.page_row = kv->d_page_table + (size_t)c.seq * g.max_pages_per_seq;
    q.len = kv->h_len[c.seq];
    q.Q = c.Q; q.ncols = c.ncols;
    q.Knew = c.Knew; q.Vnew = c.Vnew; q.n_new = c.n_new;
    q.qkv = c.qkv; q.slot0 = c.slot0;
    q.Kslot = c.Kslot; q.Vslot = c.Vslot;
    q.O = c.O;
    const int R = c.ncols * a.grp;
    const int MT = (R + 15) / 16;
    if (MT < 1 || MT > (c.full ? 5 : 3) || c.n_new > kPT || c.n_new < c.ncols || c.ncols > kMaxCols) return CAS_EINVAL;
    const int pages = (q.len + q.n_new + kPT - 1) / kPT;
    if (pages > g.max_pages_per_seq) return CAS_ENOMEM;
    q.nsplit = (pages + kPagesPerSplit - 1) / kPagesPerSplit;
    const size_t need = sizeof(float) * (size_t)q.nsplit * g.n_kv_heads * R * kPartStride;
    if (!ws || *ws_used + need > ws_bytes) return CAS_ENOMEM;
    q.part = (float*)((char*)ws + *ws_used);
    *ws_used += (need + 255) / 256 * 256;
    max_r = std::max(max_r, R);
    max_split = std::max(max_split, q.nsplit);
    // committed positions: bitmap + spec (+ lo + pruned) of K and V; in-flight ones: plain bf16
    const double per_tok = 4.0 * (4 + g.mx + g.sw + (c.full ? g.lw + g.pw : 0));
    bytes += 2.0 * g.n_kv_heads * (per_tok * q.len + 256.0 * q.n_new);
  }
  const int MT = (max_r + 15) / 16;
  dim3 grid(max_split, g.n_kv_heads, n);
  int rc;
  {
    ProfScope scope(prof ? ctx : nullptr, c0.full ? PROF_ATTN_VERIFY : PROF_ATTN_DRAFT, bytes);
    if (g.mx) {
      if (c0.full) {
        rc = MT == 1   ? launch_mt<1, true, true>(ctx, b, grid)
             : MT == 2 ? launch_mt<2, true, true>(ctx, b, grid)
             : MT == 3 ? launch_mt<3, true, true>(ctx, b, grid)
             : MT == 4 ? launch_mt<4, true, true>(ctx, b, grid)
                       : launch_mt<5, true, true>(ctx, b, grid);
      } else {
        rc = MT == 1 ? launch_mt<1, false, true>(ctx, b, grid) : MT == 2 ? launch_mt<2, false, true>(ctx, b, grid)
                                                                          : launch_mt<3, false, true>(ctx, b, grid);
      }
    } else if (c0.full) {
      rc = MT == 1   ? launch_mt<1, true>(ctx, b, grid)
           : MT == 2 ? launch_mt<2, true>(ctx, b, grid)
           : MT == 3 ? launch_mt<3, true>(ctx, b, grid)
           : MT == 4 ? launch_mt<4, true>(ctx, b, grid)
                     : launch_mt<5, true>(ctx, b, grid);
    } else {
      rc = MT == 1 ? launch_mt<1, false>(ctx, b, grid) : MT == 2 ? launch_mt<2, false>(ctx, b, grid)
                                                                  : launch_mt<3, false>(ctx, b, grid);
    }
  }
  if (rc != CAS_OK) return rc;
  hipLaunchKernelGGL(attn_merge_kernel, dim3(max_r, g.n_kv_heads, 2 * n), dim3(512),
                     sizeof(float) * (max_split + kMergeParts * 64), ctx->stream, b);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

int launch_attention_batch(cas_ctx* ctx, cas_kv* kv, const AttnCall* calls, int n) {
  if (n < 1) return CAS_OK;
  // the launches of a group follow those of the group before on the stream, so every group
  // starts at the beginning of the workspace again
  for (int i = 0; i < n; i += kAttnBatch) {
    size_t ws_used = 0;
    const int rc = launch_attention_group(ctx, kv, calls + i, std::min(kAttnBatch, n - i), ctx->d_ws, ctx->ws_bytes,
                                          &ws_used, true);
    if (rc != CAS_OK) return rc;
  }
  return CAS_OK;
}

int launch_attention(cas_ctx* ctx, cas_kv* kv, const AttnCall& c) { return launch_attention_batch(ctx, kv, &c, 1); }

// Plain bf16 attention of one decode step over an UNCOMPRESSED cache (the BFloat16 baseline, for
// context figures): the same kernels with no committed position in any pool; the cache rows play
// the part of the in-flight vectors, which the kernels take as plain bf16.  Kc, Vc:
// [max_pos][n_kv_heads][128], positions 0 .. len-1 filled; the k, v of the new token (position
// len) are split from the fp32 projection `qkv`, rotated and stored at row len.
int launch_attention_dense(cas_ctx* ctx, int n_kv_heads, int n_q_heads, uint16_t* Kc, uint16_t* Vc, int len,
                           const float* qkv, int ystride, const float* rope, uint16_t* O) {
  if (n_kv_heads < 1 || n_q_heads % n_kv_heads != 0 || len < 0 || !Kc || !Vc || !qkv || !rope || !O) return CAS_EINVAL;
  AttnBatch b{};
  AttnArgs& a = b.common;
  a.g = KvGeom{};
  a.g.n_kv_heads = n_kv_heads; a.g.page_tokens = kPT; a.g.n_pages = 1;
  a.layer = 0;
  a.n_q_heads = n_q_heads; a.grp = n_q_heads / n_kv_heads;
  a.ystride = ystride; a.rope = rope;
  a.scale = 0.08838834764831845f;
  a.pages_per_split = kPagesPerSplit;
  if (a.grp > 16) return CAS_ENOTSUP;
  AttnSeq& q = b.s[0];
  q.page_row = nullptr;  // never consulted: no position is committed to a pool
  q.len = 0; q.ncols = 1; q.n_new = len + 1; q.slot0 = len;
  q.Knew = Kc; q.Vnew = Vc; q.Kslot = Kc; q.Vslot = Vc;
  q.qkv = qkv; q.Q = nullptr; q.O = O;
  q.nsplit = (len + 1 + kPT - 1) / kPT;
  const size_t need = sizeof(float) * (size_t)q.nsplit * n_kv_heads * a.grp * kPartStride;
  if (!ctx->d_ws || need > ctx->ws_bytes) return CAS_ENOMEM;
  q.part = (float*)ctx->d_ws;
  const int rc = launch_mt<1, false>(ctx, b, dim3(q.nsplit, n_kv_heads, 1));
  if (rc != CAS_OK) return rc;
  hipLaunchKernelGGL(attn_merge_kernel, dim3(a.grp, n_kv_heads, 2), dim3(512),
                     sizeof(float) * (q.nsplit + kMergeParts * 64), ctx->stream, b);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

// ---- the variant for callers that cannot allocate: the partial results live in a fixed array of
// the library's own instead of a workspace the caller had to obtain.  Every GPU holds its own copy
// of the array at its own address; the address is looked up once per device, with that device
// current, and only that pointer (never the array's name) is handed to kernels.
constexpr size_t kAttnScratchBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kAttnScratchBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

size_t attention_static_capacity() { return kAttnScratchBytes; }

int launch_attention_static(cas_ctx* ctx, cas_kv* kv, const AttnCall& c) {
  int dev = -1;
  CAS_HIP(ctx, hipGetDevice(&dev));
  if (dev != ctx->device || dev < 0 || dev >= kMaxDevices) return CAS_EINVAL;  // the context's device must be current
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    CAS_HIP(ctx, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return CAS_EHIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // two threads racing store the same address
  }
  size_t ws_used = 0;
  // nothing in the array has to start at zero: every split writes its whole record before the
  // merge kernel, which follows on the same stream, reads exactly the records of this call
  return launch_attention_group(ctx, kv, &c, 1, ptr, kAttnScratchBytes, &ws_used, false);
}

}  // namespace cas
