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
#include "attention_kernel.inl"

namespace cas {

// the draft form (speculation data only) is compiled in attention_draft.hip
extern template int launch_mt<1, false>(cas_ctx*, const AttnArgs&, dim3);
extern template int launch_mt<2, false>(cas_ctx*, const AttnArgs&, dim3);
extern template int launch_mt<3, false>(cas_ctx*, const AttnArgs&, dim3);

// Combine the splits: o = sum_s e^{m_s - M} O_s / sum_s e^{m_s - M} l_s, rounded to bf16.
// One workgroup per (query row, kv head, half of the channels): the split weights are computed
// once into LDS, then thread (channel d, part p) sums the splits s = p, p + 8, ... with
// independent loads and the eight parts are added in part order (a fixed order: the result
// does not depend on timing, nor on how many rows ride along).
constexpr int kMergeParts = 8;
constexpr int kMergePre = 20;  // splits per thread whose outputs are requested before the weights exist
__global__ __launch_bounds__(512) void attn_merge_kernel(AttnArgs a) {
  extern __shared__ float sw[];  // [nsplit] weights, then [kMergeParts][64] partial sums
  __shared__ float red[16];
  const int rr = blockIdx.x, head = blockIdx.y, tid = threadIdx.x;
  const int d = blockIdx.z * 64 + (tid & 63), part = tid >> 6;
  const int R = a.ncols * a.grp;
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

int launch_attention(cas_ctx* ctx, cas_kv* kv, const AttnCall& c) {
  const KvGeom& g = kv->geom;
  AttnArgs a;
  a.g = g;
  a.spec_pool = (const uint32_t*)kv->d_spec;
  a.verif_pool = (const uint32_t*)kv->d_verif;
  a.page_row = kv->d_page_table + (size_t)c.seq * g.max_pages_per_seq;
  a.layer = c.layer;
  a.len = kv->h_len[c.seq];
  a.Q = c.Q; a.ncols = c.ncols; a.n_q_heads = c.n_q_heads; a.grp = c.n_q_heads / g.n_kv_heads;
  a.Knew = c.Knew; a.Vnew = c.Vnew; a.n_new = c.n_new;
  a.qkv = c.qkv; a.ystride = c.ystride; a.slot0 = c.slot0; a.rope = c.rope;
  a.Kslot = c.Kslot; a.Vslot = c.Vslot;
  a.scale = 0.08838834764831845f;  // 1 / sqrt(128)
  a.O = c.O;
  const int R = a.ncols * a.grp;
  const int MT = (R + 15) / 16;
  if (MT < 1 || MT > (c.full ? 5 : 3) || c.n_new > kPT || c.n_new < c.ncols || c.ncols > kMaxCols) return CAS_EINVAL;
  const int pages = (a.len + a.n_new + kPT - 1) / kPT;
  if (pages > g.max_pages_per_seq) return CAS_ENOMEM;
  a.pages_per_split = kPagesPerSplit;  // fixed: a query's value must not depend on the length
  a.nsplit = (pages + kPagesPerSplit - 1) / kPagesPerSplit;
  size_t need = sizeof(float) * (size_t)a.nsplit * g.n_kv_heads * R * kPartStride;
  if (need > ctx->ws_bytes || !ctx->d_ws) return CAS_ENOMEM;
  a.part = (float*)ctx->d_ws;
  dim3 grid(a.nsplit, g.n_kv_heads);
  int rc;
  {
    // committed positions: bitmap + spec (+ lo + pruned) of K and V; in-flight ones: plain bf16
    const double per_tok = 4.0 * (4 + g.sw + (c.full ? g.lw + g.pw : 0));
    const double bytes = 2.0 * g.n_kv_heads * (per_tok * a.len + 256.0 * a.n_new);
    ProfScope prof(ctx, c.full ? PROF_ATTN_VERIFY : PROF_ATTN_DRAFT, bytes);
  if (c.full) {
    rc = MT == 1   ? launch_mt<1, true>(ctx, a, grid)
         : MT == 2 ? launch_mt<2, true>(ctx, a, grid)
         : MT == 3 ? launch_mt<3, true>(ctx, a, grid)
         : MT == 4 ? launch_mt<4, true>(ctx, a, grid)
                   : launch_mt<5, true>(ctx, a, grid);
  } else {
    rc = MT == 1 ? launch_mt<1, false>(ctx, a, grid) : MT == 2 ? launch_mt<2, false>(ctx, a, grid)
                                                                : launch_mt<3, false>(ctx, a, grid);
  }
  }
  if (rc != CAS_OK) return rc;
  hipLaunchKernelGGL(attn_merge_kernel, dim3(R, g.n_kv_heads, 2), dim3(512), sizeof(float) * (a.nsplit + kMergeParts * 64),
                     ctx->stream, a);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

}  // namespace cas
