// Kernel template and launcher of the verification GEMM; gemm_verify.hip instantiates the forms
// for up to 8 columns, gemm_verify_wide.hip those for 9 to 32.
#pragma once
#include <algorithm>
#include "cas_device.hpp"
#include "cas_internal.hpp"

namespace cas {

typedef short bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct VerifyArgs {
  int rows, cols, bw, sw, lw, pw, ncols;
  const uint32_t* bitmap;
  const uint32_t* spec;
  const uint32_t* lo;
  const uint32_t* pruned;
  const uint16_t* X;  // [ncols][cols]
  float* Y;           // [ncols][yld] (epilogue 0)
  int yld;            // output rows per column in Y / out16 (>= rows: the launch may cover a block of rows)
  const uint8_t* sexp;  // shared-exponent form only: one exponent per bitmap word, ew bytes per row
  int ew;
  int epi;            // 0: Y = W X;  1: h = bf16(h + bf16(W X));  2: act[i] = swiglu(rows 2i, 2i+1)
  uint16_t* out16;    // h [ncols][yld] (epilogue 1) or act [ncols][yld/2] (epilogue 2)
};

constexpr int kSlabCols = 2048;
// row groups below which a matrix gets more waves per row group (just over one group per CU)
constexpr int kFewGroups = 300;
constexpr int kGroupPitch = 36;         // 4 dump slots + 32 columns
constexpr int kTilePitch = 148;         // 4 groups + 4 pad, keeps 8-byte alignment, spreads banks

// G row groups of 16 rows per workgroup, each split over Q waves that take 2048/Q columns of
// every slab.  XST: decode steps per staging of X (a wave stages the X columns of its next XST
// steps; fewer steps = less LDS per wave, which keeps several workgroups per CU when there are
// many columns).  NB: blocks of 16 output columns (MFMA N = 16); every column is computed by
// the same operations whichever block and whatever company it has.  At decode step i the four lanes (r, 0..3) of a row take four CONSECUTIVE bitmap
// words, so one step reads one contiguous run of each stream per row and every cache line is
// fetched by one step only (lines are not kept in L1 between steps: 12 waves x 16 rows x 3
// streams are far more than it holds).
template <int T, int G, int Q, int XST, int NB, bool MX = false>
__global__ __launch_bounds__(64 * G * Q) void gemm_verify_kernel(VerifyArgs a) {
  constexpr int NW = G * Q;          // waves per workgroup
  constexpr int NT = 64 * NW;        // threads
  constexpr int WPP = 64 / Q;        // bitmap words per part and slab
  constexpr int WPL = WPP / 4;       // words per lane and slab = decode steps per slab
  static_assert(WPL >= 1, "at most 16 parts");
  static_assert(XST >= 1 && WPL % XST == 0 && NB >= 1 && NB <= 2, "staging divides the steps of a slab");
  constexpr int XQ = XST * 128;      // X columns one wave stages at a time
  constexpr int XQP = XQ + 8;        // row pitch of its private copy (bf16)
  extern __shared__ uint16_t lds[];
  uint16_t* tiles = lds;                                 // [NW][16][kTilePitch]
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int gi = wv / Q, part = wv % Q;
  uint16_t* tile = tiles + wv * 16 * kTilePitch;
  uint16_t* Xq = lds + NW * 16 * kTilePitch + (size_t)wv * a.ncols * XQP;  // [ncols][XQP], this wave's
  // columns past the end of a ragged row are never written by the decode: they must read as 0
  for (int i = tid; i < NW * 16 * kTilePitch / 8; i += NT) reinterpret_cast<uint4*>(tiles)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();

  const int r = lane >> 2, j = lane & 3;
  const int row0 = (blockIdx.x * G + gi) * 16;
  const int row = min(row0 + r, a.rows - 1);
  const uint32_t* bm_row = a.bitmap + (size_t)row * a.bw;
  const uint32_t* sp_row = a.spec + (size_t)row * a.sw;
  const uint32_t* lo_row = a.lo + (size_t)row * a.lw;
  const uint32_t* pr_row = a.pruned + (size_t)row * a.pw;
  uint16_t* trow = tile + r * kTilePitch + j * kGroupPitch + 4;  // column 0 of the lane's group

  // MFMA operand addresses: A[i = lane%16][k = 4*(lane/16)..+3], B[k][n = lane%16]
  const int mi = lane & 15, mq = lane >> 4;
  const uint16_t* a_base = tile + mi * kTilePitch + 4 + 4 * mq;
  const uint16_t* b_base[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) b_base[nb] = Xq + (16 * nb + mi < a.ncols ? 16 * nb + mi : 0) * XQP + 4 * mq;
  const bool xvec = (a.cols & 7) == 0;  // 16-byte pieces of X rows are aligned and never straddle the end

  f32x4 C[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) C[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  uint32_t rowpre = 0;  // kept values of the row in earlier slabs
  const int nslab = (a.bw + 63) >> 6;

  // bitmap words of a slab: for every part v, this lane's words v*WPP + 4*i + j
  uint32_t mw[Q][WPL];
  auto load_bitmaps = [&](int slab) {
#pragma unroll
    for (int v = 0; v < Q; ++v) {
      int w0 = slab * 64 + v * WPP + j;
#pragma unroll
      for (int i = 0; i < WPL; ++i) mw[v][i] = (w0 + 4 * i < a.bw) ? bm_row[w0 + 4 * i] : 0u;
    }
  };
  load_bitmaps(0);

  for (int slab = 0; slab < nslab; ++slab) {
    // ---- kept values of the row before this wave's part, then before each of this lane's words
    uint32_t before = rowpre;
    int slab_total = 0;
    uint32_t m4[WPL];
#pragma unroll
    for (int v = 0; v < Q; ++v) {
      int cq = 0;
#pragma unroll
      for (int i = 0; i < WPL; ++i) cq += __popc(mw[v][i]);
      int s = cq;
      s += quad_dpp<0xB1>(s);  // quad_perm [1,0,3,2]
      s += quad_dpp<0x4E>(s);  // quad_perm [2,3,0,1]
      slab_total += s;
      if (v < part) before += (uint32_t)s;
      if (v == part) {
#pragma unroll
        for (int i = 0; i < WPL; ++i) m4[i] = mw[v][i];
      }
    }
    rowpre += (uint32_t)slab_total;
    if (slab + 1 < nslab) load_bitmaps(slab + 1);  // in flight while this slab is decoded

    // per word: kept / pruned masks and the positions of its first fields in the streams
    const int word0 = slab * 64 + part * WPP + j;
    uint32_t pm4[WPL], p4[WPL], u4[WPL];
    {
      uint32_t pstep = before;  // kept values before the four words of step i
#pragma unroll
      for (int i = 0; i < WPL; ++i) {
        const int cnt = __popc(m4[i]);
        const int b0 = quad_dpp<0x00>(cnt), b1 = quad_dpp<0x55>(cnt), b2 = quad_dpp<0xAA>(cnt), b3 = quad_dpp<0xFF>(cnt);
        const uint32_t p = pstep + (uint32_t)((j > 0 ? b0 : 0) + (j > 1 ? b1 : 0) + (j > 2 ? b2 : 0));
        pstep += (uint32_t)(b0 + b1 + b2 + b3);
        const int nvalid = a.cols - (word0 + 4 * i) * 32;
        const uint32_t valid = nvalid >= 32 ? 0xFFFFFFFFu : (nvalid <= 0 ? 0u : ((1u << nvalid) - 1u));
        pm4[i] = ~m4[i] & valid;
        // words past the end of the row have no fields: keep their (unused) windows in range
        p4[i] = nvalid > 0 ? p : 0u;
        u4[i] = nvalid > 0 ? (uint32_t)(word0 + 4 * i) * 32u - p : 0u;
      }
    }
    // shared-exponent form: the exponent of each of the lane's words (sp_row is then the field stream)
    int E4[WPL];
    if constexpr (MX) {
#pragma unroll
      for (int i = 0; i < WPL; ++i)
        E4[i] = word0 + 4 * i < a.bw ? (int)a.sexp[(size_t)row * a.ew + word0 + 4 * i] : 0;
    }
    KeptWindows<T, true, MX> kw;
    PrunedWindows pw;
    kw.load(p4[0], sp_row, lo_row);
    // ---- this wave's X columns of the next XST steps (bf16, zero beyond the last column)
    auto stage_x = [&](int s) {
      const int col0 = slab * kSlabCols + part * (WPP * 32) + s * XQ;
      if (xvec) {
        for (int i = lane; i < a.ncols * (XQ / 8); i += 64) {
          int c = i / (XQ / 8), o = (i - c * (XQ / 8)) * 8;
          uint4 v = make_uint4(0, 0, 0, 0);
          if (col0 + o < a.cols) v = *reinterpret_cast<const uint4*>(a.X + (size_t)c * a.cols + col0 + o);
          *reinterpret_cast<uint4*>(Xq + c * XQP + o) = v;
        }
      } else {
        for (int c = 0; c < a.ncols; ++c)
          for (int i = lane; i < XQ; i += 64)
            Xq[c * XQP + i] = col0 + i < a.cols ? a.X[(size_t)c * a.cols + col0 + i] : (uint16_t)0;
      }
    };

    static_for<0, WPL>([&](auto I) {
      constexpr int i = decltype(I)::value;
      // the MFMA reads of the previous staging ended with the fence that closes a step
      if constexpr (i % XST == 0) stage_x(i / XST);
      // Half-step pipeline: the pruned values of this step are fetched while its kept values
      // are placed, the kept fields of the next step while the pruned values are placed.  One
      // raw window set of each kind is live at a time (116 registers instead of 156 with two
      // whole sets); measured 4 % faster than loading a whole step ahead.
      // pos == -1 (lane out of bits) lands in the dump slot in front of the group
      pw.load(u4[i], pr_row);
      kw.decode(m4[i], [&](int pos, uint16_t v) { trow[pos] = v; }, MX ? E4[i] : 0);
      if constexpr (i + 1 < WPL) kw.load(p4[i + 1], sp_row, lo_row);
      pw.decode(pm4[i], [&](int pos, uint16_t v) { trow[pos] = v; });
      // ---- tile x X: tile column 32*g + c is slab column (part*WPP + 4*i + g)*32 + c
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const int g = kk >> 1, h = kk & 1;
        bf16x4 av = *reinterpret_cast<const bf16x4*>(a_base + g * kGroupPitch + h * 16);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          bf16x4 bv = *reinterpret_cast<const bf16x4*>(b_base[nb] + (4 * (i % XST) + g) * 32 + h * 16);
          C[nb] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, bv, C[nb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    });
  }

  // ---- add the Q partial tiles of each row group in part order; C[i][n]: i = 4*(lane/16) + e, n = lane%16
  __syncthreads();
  float* red = reinterpret_cast<float*>(lds);  // [NB][NW][64][4], reuses the tiles
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) *reinterpret_cast<f32x4*>(red + ((nb * NW + wv) * 64 + lane) * 4) = C[nb];
  __syncthreads();
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int col = 16 * nb + mi;
    if (part != 0 || col >= a.ncols) continue;
    f32x4 s = *reinterpret_cast<f32x4*>(red + ((nb * NW + wv) * 64 + lane) * 4);
#pragma unroll
    for (int w = 1; w < Q; ++w) s += *reinterpret_cast<f32x4*>(red + ((nb * NW + wv + w) * 64 + lane) * 4);
    if (a.epi == 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int orow = row0 + 4 * mq + e;
        if (orow < a.rows) a.Y[(size_t)col * a.yld + orow] = s[e];
      }
    } else if (a.epi == 1) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int orow = row0 + 4 * mq + e;
        if (orow < a.rows) {
          uint16_t* hp = a.out16 + (size_t)col * a.yld + orow;
          *hp = f32_to_bf16(bf16_to_f32(*hp) + round_bf16(s[e]));
        }
      }
    } else {  // rows come in (gate, up) pairs; a lane holds rows 4*mq .. 4*mq+3 = two pairs
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        int orow = row0 + 4 * mq + e;
        if (orow + 1 < a.rows) {
          const float g = round_bf16(s[e]), u = round_bf16(s[e + 1]);
          a.out16[(size_t)col * (a.yld >> 1) + (orow >> 1)] = f32_to_bf16(g / (1.0f + expf(-g)) * u);
        }
      }
    }
  }
}

template <int G, int Q, int XST, int NB, bool MX = false>
static int launch_gq(cas_ctx* ctx, const VerifyArgs& a, int t) {
  constexpr int NW = G * Q;
  size_t lds = sizeof(uint16_t) * (NW * 16 * kTilePitch + (size_t)NW * a.ncols * (XST * 128 + 8));
  lds = std::max(lds, sizeof(float) * NB * NW * 64 * 4);
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  const int groups = (a.rows + 15) / 16;
  const int grid = (groups + G - 1) / G;
#define CAS_LAUNCH(TV)                                                                                        \
  case TV: {                                                                                                  \
    static LdsLimit lim;                                                                                      \
    const int rc = allow_lds(ctx, (const void*)gemm_verify_kernel<TV, G, Q, XST, NB, MX>, lds, lim);              \
    if (rc != CAS_OK) return rc;                                                                              \
    hipLaunchKernelGGL((gemm_verify_kernel<TV, G, Q, XST, NB, MX>), dim3(grid), dim3(64 * NW), lds, ctx->stream, a); \
  } break;
  switch (t) {
    CAS_LAUNCH(0) CAS_LAUNCH(1) CAS_LAUNCH(2) CAS_LAUNCH(3) CAS_LAUNCH(4) CAS_LAUNCH(5) CAS_LAUNCH(6) CAS_LAUNCH(7)
    default: return CAS_EINVAL;
  }
#undef CAS_LAUNCH
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

// ---- which form of the kernel a matrix gets ----------------------------------------------------
// The choice depends on the shape of the WHOLE matrix (a.yld rows), never on the number of columns
// or on the block of rows a launch covers: it fixes the order in which a row's partial sums are
// added, and a column must get the same bits in every call.

// Up to 8 columns.  One row group per workgroup.  Many row groups: four waves, each taking a
// quarter of every slab (measured faster than 8-wave workgroups: fewer lanes wait at the slab
// barriers).  Few row groups: eight waves so that every CU still gets several, sixteen when the
// rows are long (each wave then has one decode step per slab and the serial chain per workgroup
// halves).  X is staged per slab: measured 5 % faster on the largest matrices than per step.
template <bool MX>
static int verify_narrow(cas_ctx* ctx, const VerifyArgs& a, int t) {
  const int groups = (a.yld + 15) / 16;
  if (groups < kFewGroups && a.cols >= 4 * kSlabCols) return launch_gq<1, 16, 1, 1, MX>(ctx, a, t);
  if (groups < kFewGroups) return launch_gq<1, 8, 2, 1, MX>(ctx, a, t);
  return launch_gq<1, 4, 4, 1, MX>(ctx, a, t);
}

// 9 to 32 columns (several sequences per pass, or long drafts): X staged one decode step at a
// time, so that the LDS of a workgroup stays small enough for three of them per CU, and a second
// block of 16 output columns above 16.
template <int NB, bool MX>
static int verify_wide_nb(cas_ctx* ctx, const VerifyArgs& a, int t) {
  const int groups = (a.yld + 15) / 16;
  if (groups < kFewGroups && a.cols >= 4 * kSlabCols) return launch_gq<1, 16, 1, NB, MX>(ctx, a, t);
  if (groups < kFewGroups) return launch_gq<1, 8, 1, NB, MX>(ctx, a, t);
  return launch_gq<1, 4, 1, NB, MX>(ctx, a, t);
}

template <bool MX>
static int verify_wide(cas_ctx* ctx, const VerifyArgs& a, int t) {
  if (a.ncols <= 16) return verify_wide_nb<1, MX>(ctx, a, t);
  int rc = verify_wide_nb<2, MX>(ctx, a, t);
  if (rc != CAS_ENOTSUP) return rc;
  // sixteen waves per row group with more than 20 columns exceed the LDS: two launches of one
  // column block each (the weights of such a matrix are read twice)
  VerifyArgs lo = a, hi = a;
  lo.ncols = 16;
  hi.ncols = a.ncols - 16;
  hi.X = a.X + (size_t)16 * a.cols;
  if (a.Y) hi.Y = a.Y + (size_t)16 * a.yld;
  if (a.out16) hi.out16 = a.out16 + (size_t)16 * (a.epi == 2 ? a.yld >> 1 : a.yld);
  rc = verify_wide_nb<1, MX>(ctx, lo, t);
  if (rc != CAS_OK) return rc;
  return verify_wide_nb<1, MX>(ctx, hi, t);
}

// gemm_verify_wide.hip: verify_wide<false> (its own translation unit: the build compiles the files side by side)
int launch_gemm_verify_wide(cas_ctx* ctx, const VerifyArgs& a, int t);

}  // namespace cas
