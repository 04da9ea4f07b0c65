// Partial attention kernel over one page of the compressed cache and its launcher, compiled
// in two translation units (exact form / draft form); attention.hip explains the algorithm.
#pragma once
#include "cas_device.hpp"
#include "cas_internal.hpp"

namespace cas {

typedef short bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct AttnArgs {
  KvGeom g;
  const uint32_t* spec_pool;
  const uint32_t* verif_pool;
  const int32_t* page_row;  // page table row of the sequence
  int layer, len, nsplit, pages_per_split;
  const uint16_t* Q;
  int ncols, n_q_heads, grp;  // grp = query heads per kv head
  const uint16_t* Knew;
  const uint16_t* Vnew;
  int n_new;
  // fused split of the qkv projection (model path): when qkv != null the columns' q, k, v are
  // taken from the fp32 projection output, rounded to bf16 and rotated here, and the k, v of
  // the columns are also written to their in-flight slots for later passes and the commit
  const float* qkv;   // [ncols][ystride]: q heads, k heads, v heads
  int ystride, slot0; // slot0: in-flight slot of column 0 (its position is len + slot0)
  const float* rope;  // [max_pos][64][2] cos, sin
  uint16_t* Kslot;    // writable views of Knew / Vnew
  uint16_t* Vslot;
  float scale;
  float* part;  // [nsplit][n_kv_heads][R][132]
  uint16_t* O;
};

// What differs between the sequences of one launch; blockIdx.z picks the sequence.
constexpr int kAttnBatch = 4;
struct AttnSeq {
  const int32_t* page_row;
  int len, nsplit, ncols, n_new, slot0;
  const uint16_t* Q;
  const uint16_t* Knew;
  const uint16_t* Vnew;
  const float* qkv;
  uint16_t* Kslot;
  uint16_t* Vslot;
  float* part;
  uint16_t* O;
};
struct AttnBatch {
  AttnArgs common;  // its per-sequence members are filled in from s[] inside the kernels
  AttnSeq s[kAttnBatch];
};
__device__ __forceinline__ AttnArgs attn_args_of(const AttnBatch& b, int z) {
  AttnArgs a = b.common;
  const AttnSeq& q = b.s[z];
  a.page_row = q.page_row; a.len = q.len; a.nsplit = q.nsplit; a.ncols = q.ncols; a.n_new = q.n_new;
  a.slot0 = q.slot0; a.Q = q.Q; a.Knew = q.Knew; a.Vnew = q.Vnew; a.qkv = q.qkv;
  a.Kslot = q.Kslot; a.Vslot = q.Vslot; a.part = q.part; a.O = q.O;
  return a;
}

constexpr int kPT = 64;          // tokens per page
constexpr int kQP = 136;         // Q row pitch (bf16)
constexpr int kKG = 36, kKP = 148;  // K tile: group pitch (4 dump + 32), row pitch
constexpr int kVP = 72;          // transposed V tile: token pitch per channel row
constexpr int kVR = 132;         // channel rows: 4 groups x (1 dump + 32)
constexpr int kPP = 72;          // probability row pitch (bf16)
constexpr int kPartStride = 132;
constexpr int kPagesPerSplit = 1;
constexpr int kMaxCols = 16;     // columns of one pass whose k, v may be split from the projection here

constexpr int kKVTile = kPT * kKP > kVR * kVP ? kPT * kKP : kVR * kVP;  // K and V^T tiles share one region
constexpr int kQPRows = kQP > 2 * kPP ? kQP : 2 * kPP;                  // Q and (P head, P remainder) share one region

template <int MT>
constexpr size_t attn_lds_bytes() {
  return sizeof(uint16_t) * (MT * 16 * kQPRows + kKVTile) + sizeof(float) * (8 * MT * 16);
}

// all-reduce over the 16 lanes of a DPP row by rotations; every lane ends with the result
template <int CTRL>
__device__ __forceinline__ float row_rot(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, row_rot<0x121>(v));
  v = fmaxf(v, row_rot<0x122>(v));
  v = fmaxf(v, row_rot<0x124>(v));
  return fmaxf(v, row_rot<0x128>(v));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += row_rot<0x121>(v);
  v += row_rot<0x122>(v);
  v += row_rot<0x124>(v);
  return v + row_rot<0x128>(v);
}

// MX: the cache is in the shared-exponent form (one exponent per 32-channel block of a vector)
template <int MT, bool FULL, int T, bool MX = false>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnBatch batch) {
  const AttnArgs a = attn_args_of(batch, blockIdx.z);
  if ((int)blockIdx.x >= a.nsplit) return;  // a shorter sequence of the launch: uniform for the workgroup
  extern __shared__ uint16_t lds16[];
  uint16_t* Qs = lds16;                       // [MT*16][kQP]; dead once the scores are in registers
  uint16_t* Ph = lds16;                       // [MT*16][kPP] over the Q region
  uint16_t* Pl = Ph + MT * 16 * kPP;          // [MT*16][kPP]
  uint16_t* Kt = lds16 + MT * 16 * kQPRows;   // [64][kKP]
  uint16_t* Vt = Kt;                          // [kVR][kVP]: the K tile is dead once the scores are out
  float* wm = reinterpret_cast<float*>(Kt + kKVTile);  // [4 waves][MT*16] row maximum over the wave's 16 tokens
  float* wl = wm + 4 * MT * 16;                        // [4 waves][MT*16] row sum of exponentials

  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pg = blockIdx.x, head = blockIdx.y;  // one page (64 positions) per workgroup
  const int R = a.ncols * a.grp;
  const KvGeom& g = a.g;
  const int r = tid >> 2, j = tid & 3;           // decode role: token r of the page, word j
  const int mi = lane & 15, mq = lane >> 4;      // MFMA role
  uint16_t* krow = Kt + r * kKP + j * kKG + 4;
  uint16_t* vcol = Vt + (33 * j + 1) * kVP + r;

  const int total = a.len + a.n_new;             // committed + in-flight positions
  const int tok0 = pg * kPT;
  const int ntok = min(kPT, total - tok0);
  const int pos = tok0 + r;                      // position of this thread's token
  const bool live = pos < a.len;                 // committed: decode from the cache
  const bool fresh = !live && pos < total;       // in flight: uncompressed vector
  const int first = a.len + a.slot0;             // position of column 0 of this pass
  // in flight and produced by this very pass: split from the projection below by all threads
  const bool own_new = a.qkv != nullptr && fresh && pos >= first;
  // the page table is consulted only for pages that hold committed positions: a page of in-flight
  // positions alone needs no pool page yet (and the plain-bf16 form has no pool at all)
  const int page = tok0 < a.len ? min(max(a.page_row[pg], 0), g.n_pages - 1) : 0;

  // ---- 0. loads that do not depend on the page table entry go out first: the queries and,
  //         in the fused form, the k, v of this pass's columns that fall into this page
  constexpr int NQ = MT * 4;
  float x0[NQ], x1[NQ], cc[NQ], sn[NQ];
  uint4 qraw[MT];
  // fused k, v split: thread (column cf of a batch of 8, channel quarter dq) handles channels
  // dq, dq+32 and their rotation partners dq+64, dq+96
  const int cf = tid >> 5, dq = tid & 31;
  float kx[2][4], vx[2][4];
  float2 kcs[2][2];
  bool fnew[2];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const int c = cb * 8 + cf, fpos = first + c;
    fnew[cb] = a.qkv != nullptr && c < a.ncols && fpos >= tok0 && fpos < tok0 + kPT;
  }
  if (a.qkv) {
#pragma unroll
    for (int it = 0; it < NQ; ++it) {
      const int i = tid + it * 256, rr = i >> 6, d = i & 63;
      x0[it] = x1[it] = cc[it] = sn[it] = 0.f;
      if (rr < R) {
        const int c = rr / a.grp, gi = rr - c * a.grp;
        const float* src = a.qkv + (size_t)c * a.ystride + (size_t)(head * a.grp + gi) * 128;
        const float2 cs = *reinterpret_cast<const float2*>(a.rope + ((size_t)(first + c) * 64 + d) * 2);
        x0[it] = src[d]; x1[it] = src[d + 64]; cc[it] = cs.x; sn[it] = cs.y;
      }
    }
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      if (fnew[cb]) {
        const int c = cb * 8 + cf;
        const float* src = a.qkv + (size_t)c * a.ystride + (size_t)(a.n_q_heads + head) * 128;
        const float* vsrc = src + (size_t)g.n_kv_heads * 128;
        const float* cs = a.rope + (size_t)(first + c) * 128;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          kx[cb][q] = src[dq + 32 * q];
          vx[cb][q] = vsrc[dq + 32 * q];
        }
        kcs[cb][0] = *reinterpret_cast<const float2*>(cs + 2 * dq);
        kcs[cb][1] = *reinterpret_cast<const float2*>(cs + 2 * (dq + 32));
      }
    }
  } else {
#pragma unroll
    for (int it = 0; it < MT; ++it) {  // 16-byte pieces
      const int i = tid + it * 256, rr = i >> 4, d = (i & 15) * 8;
      qraw[it] = make_uint4(0, 0, 0, 0);
      if (rr < R) {
        const int c = rr / a.grp, gi = rr - c * a.grp;
        qraw[it] = *reinterpret_cast<const uint4*>(a.Q + ((size_t)c * a.n_q_heads + head * a.grp + gi) * 128 + d);
      }
    }
  }

  // ---- 1. bitmap words of this thread's (token, word) of K and V; the queries are converted
  //         while they are in flight, then the stream windows are requested
  const size_t tk = (((size_t)a.layer * g.n_pages + page) * 2 + 0) * g.n_kv_heads + head;
  const size_t tv = tk + g.n_kv_heads;
  const uint32_t* ks = a.spec_pool + tk * g.tile_spec_words;
  const uint32_t* vs = a.spec_pool + tv * g.tile_spec_words;
  const uint32_t* kvf = a.verif_pool + tk * g.tile_verif_words;
  const uint32_t* vvf = a.verif_pool + tv * g.tile_verif_words;
  const uint32_t mk = live ? ks[r * 4 + j] : 0u;
  const uint32_t mv = live ? vs[r * 4 + j] : 0u;
  int ek = 0, ev = 0;  // shared-exponent form: exponent of this thread's block (byte j of the token's word)
  if constexpr (MX) {
    if (live) {
      ek = (int)((ks[kPT * 4 + r] >> (8 * j)) & 0xFFu);
      ev = (int)((vs[kPT * 4 + r] >> (8 * j)) & 0xFFu);
    }
  }
  // ---- 2. queries to LDS: row rr = column * grp + member; rows past R are 0
  if (a.qkv) {
#pragma unroll
    for (int it = 0; it < NQ; ++it) {
      const int i = tid + it * 256, rr = i >> 6, d = i & 63;
      const float a0 = round_bf16(x0[it]), a1 = round_bf16(x1[it]);
      Qs[rr * kQP + d] = f32_to_bf16(a0 * cc[it] - a1 * sn[it]);
      Qs[rr * kQP + d + 64] = f32_to_bf16(a1 * cc[it] + a0 * sn[it]);
    }
  } else {
#pragma unroll
    for (int it = 0; it < MT; ++it) {
      const int i = tid + it * 256, rr = i >> 4, d = (i & 15) * 8;
      *reinterpret_cast<uint4*>(Qs + rr * kQP + d) = qraw[it];
    }
  }
  WordWindows<T, FULL, MX> wk, wvw;
  auto word_prefix = [&](uint32_t m) -> uint32_t {  // kept values of the token before word j
    const int cnt = __popc(m);
    const int b0 = quad_dpp<0x00>(cnt), b1 = quad_dpp<0x55>(cnt), b2 = quad_dpp<0xAA>(cnt);
    return (uint32_t)((j > 0 ? b0 : 0) + (j > 1 ? b1 : 0) + (j > 2 ? b2 : 0));
  };
  // the pools are touched only by workgroups whose page holds committed positions (uniform for the
  // workgroup): such a page has a tile of its own, so the rows of its not yet committed tokens can
  // be read as well (their masks are 0 and the decode never looks at their windows)
  const bool has_live = tok0 < a.len;
  auto load_v = [&]() {
    const uint32_t p = word_prefix(mv);
    if (has_live) wvw.load(p, 32u * j - p, vs + g.spec_off + r * g.sw, vvf + r * g.lw, vvf + kPT * g.lw + r * g.pw);
  };
  {
    const uint32_t p = word_prefix(mk);
    if (has_live) wk.load(p, 32u * j - p, ks + g.spec_off + r * g.sw, kvf + r * g.lw, kvf + kPT * g.lw + r * g.pw);
  }
  // the draft form has registers to spare for both windows; the exact form asks for V later
  if constexpr (!FULL) load_v();

  // k, v of this pass's columns: round, rotate k; k goes straight into its tile row, v waits
  // in registers until the tile region is free; both go to their in-flight slots
  uint16_t fv[2][4];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    if (fnew[cb]) {
      const int c = cb * 8 + cf, fpos = first + c;
      uint16_t* kdst = Kt + (fpos - tok0) * kKP + 4;
      const size_t so = ((size_t)(fpos - a.len) * g.n_kv_heads + head) * 128;
#pragma unroll
      for (int h = 0; h < 2; ++h) {  // channel pair (dq + 32h, dq + 32h + 64)
        const float a0 = round_bf16(kx[cb][h]), a1 = round_bf16(kx[cb][h + 2]);
        const uint16_t k0 = f32_to_bf16(a0 * kcs[cb][h].x - a1 * kcs[cb][h].y);
        const uint16_t k1 = f32_to_bf16(a1 * kcs[cb][h].x + a0 * kcs[cb][h].y);
        kdst[h * kKG + dq] = k0;
        kdst[(h + 2) * kKG + dq] = k1;
        a.Kslot[so + dq + 32 * h] = k0;
        a.Kslot[so + dq + 32 * h + 64] = k1;
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        fv[cb][q] = f32_to_bf16(vx[cb][q]);
        a.Vslot[so + dq + 32 * q] = fv[cb][q];
      }
    }
  }
  __syncthreads();

  // ---- 3. K tile: this thread's 32 channels of its token
  {
    if (!own_new) {
#pragma unroll
      for (int q = 0; q < 8; ++q) *reinterpret_cast<uint64_t*>(krow + 4 * q) = 0ull;
      if (fresh) {
        const uint16_t* src = a.Knew + ((size_t)(pos - a.len) * g.n_kv_heads + head) * 128 + 32 * j;
#pragma unroll
        for (int q = 0; q < 8; ++q)
          *reinterpret_cast<uint64_t*>(krow + 4 * q) = *reinterpret_cast<const uint64_t*>(src + 4 * q);
      }
    }
    wk.decode(mk, (FULL && live) ? ~mk : 0u, [&](int bp, uint16_t v) { krow[bp] = v; }, ek);
  }
  if constexpr (FULL) load_v();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  // ---- 4. scores of this wave's 16 tokens against all query rows, kept in registers:
  //         lane (mi, mq) holds token 16 wv + mi of rows mt*16 + 4 mq + e
  float sc[MT][4];
  {
    const uint16_t* b_base = Kt + (16 * wv + mi) * kKP + 4 + 4 * mq;
    const int t = 16 * wv + mi;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      f32x4 C = {0.f, 0.f, 0.f, 0.f};
      const uint16_t* a_base = Qs + (mt * 16 + mi) * kQP + 4 * mq;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        bf16x4 av = *reinterpret_cast<const bf16x4*>(a_base + kk * 16);
        bf16x4 bv = *reinterpret_cast<const bf16x4*>(b_base + (kk >> 1) * kKG + (kk & 1) * 16);
        C = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bv, C, 0, 0, 0);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int rr = mt * 16 + 4 * mq + e;
        // column c sees positions 0 .. len + n_new - ncols + c
        const int c = rr / a.grp;
        const bool ok = t < ntok && (tok0 + t <= total - a.ncols + c);
        sc[mt][e] = ok ? C[e] * a.scale : -INFINITY;
        const float mx = row16_max(sc[mt][e]);
        if (mi == 0) wm[wv * (MT * 16) + rr] = mx;
      }
    }
  }
  __syncthreads();  // every wave is done with Q and K: their regions may be overwritten
  // ---- 5. softmax numerators of the page, head + remainder in bf16; row sums per wave
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int rr = mt * 16 + 4 * mq + e, t = 16 * wv + mi;
      const float mx = fmaxf(fmaxf(wm[rr], wm[MT * 16 + rr]), fmaxf(wm[2 * MT * 16 + rr], wm[3 * MT * 16 + rr]));
      const float p = (sc[mt][e] == -INFINITY) ? 0.f : __expf(sc[mt][e] - mx);
      const uint16_t ph = f32_to_bf16(p);
      Ph[rr * kPP + t] = ph;
      Pl[rr * kPP + t] = f32_to_bf16(p - bf16_to_f32(ph));
      const float ps = row16_sum(p);
      if (mi == 0) wl[wv * (MT * 16) + rr] = ps;
    }
  }
  // ---- 6. V tile, transposed: Vt[channel][token]
  {
    if (!own_new) {
#pragma unroll
      for (int c = 0; c < 32; ++c) vcol[c * kVP] = 0;
      if (fresh) {
        const uint16_t* src = a.Vnew + ((size_t)(pos - a.len) * g.n_kv_heads + head) * 128 + 32 * j;
#pragma unroll
        for (int c = 0; c < 32; ++c) vcol[c * kVP] = src[c];
      }
    }
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      if (fnew[cb]) {
        const int tr = first + cb * 8 + cf - tok0;
#pragma unroll
        for (int q = 0; q < 4; ++q) Vt[(33 * q + 1 + dq) * kVP + tr] = fv[cb][q];
      }
    }
    wvw.decode(mv, (FULL && live) ? ~mv : 0u, [&](int bp, uint16_t v) { vcol[bp * kVP] = v; }, ev);
  }
  __syncthreads();
  // ---- 7. O = P V ; wave w owns channels 32w .. 32w+31; partial result of this page
  float* part = a.part + ((size_t)pg * g.n_kv_heads + head) * R * kPartStride;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      f32x4 C = {0.f, 0.f, 0.f, 0.f};
      const uint16_t* b_base = Vt + (33 * wv + 1 + nt * 16 + mi) * kVP + 4 * mq;
      const uint16_t* ah = Ph + (mt * 16 + mi) * kPP + 4 * mq;
      const uint16_t* al = Pl + (mt * 16 + mi) * kPP + 4 * mq;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        bf16x4 bv = *reinterpret_cast<const bf16x4*>(b_base + kb * 16);
        C = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(*reinterpret_cast<const bf16x4*>(ah + kb * 16), bv, C, 0, 0, 0);
        C = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(*reinterpret_cast<const bf16x4*>(al + kb * 16), bv, C, 0, 0, 0);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int rr = mt * 16 + 4 * mq + e;
        if (rr < R) part[rr * kPartStride + 32 * wv + nt * 16 + mi] = C[e];
      }
    }
  }
  if (tid < R) {
    const float* m4 = wm + tid;
    const float* l4 = wl + tid;
    part[tid * kPartStride + 128] = fmaxf(fmaxf(m4[0], m4[MT * 16]), fmaxf(m4[2 * MT * 16], m4[3 * MT * 16]));
    part[tid * kPartStride + 129] = ((l4[0] + l4[MT * 16]) + l4[2 * MT * 16]) + l4[3 * MT * 16];
  }
}

template <int MT, bool FULL, bool MX = false>
int launch_mt(cas_ctx* ctx, const AttnBatch& a, dim3 grid) {
  constexpr size_t lds = attn_lds_bytes<MT>();
#define CAS_LAUNCH(TV)                                                                                     \
  case TV: {                                                                                               \
    static LdsLimit lim;                                                                                   \
    const int rc = allow_lds(ctx, (const void*)attn_partial_kernel<MT, FULL, TV, MX>, lds, lim);               \
    if (rc != CAS_OK) return rc;                                                                           \
    hipLaunchKernelGGL((attn_partial_kernel<MT, FULL, TV, MX>), grid, dim3(256), lds, ctx->stream, a);         \
  } break;
  switch (a.common.g.t) {
    CAS_LAUNCH(0) CAS_LAUNCH(1) CAS_LAUNCH(2) CAS_LAUNCH(3) CAS_LAUNCH(4) CAS_LAUNCH(5) CAS_LAUNCH(6) CAS_LAUNCH(7)
    default: return CAS_EINVAL;
  }
#undef CAS_LAUNCH
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

}  // namespace cas
