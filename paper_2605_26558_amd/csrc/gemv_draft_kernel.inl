// Kernel template of the draft GEMV, shared by the raw-exponent form (gemv_draft.hip) and the
// shared-exponent form (mx.hip); each of the two files instantiates its own set.
#pragma once
#include <algorithm>
#include "cas_device.hpp"
#include "cas_internal.hpp"

namespace cas {

struct GemvArgs {
  int rows, cols, bw, sw, nwaves;
  const uint32_t* bitmap;
  const uint32_t* spec;
  const uint16_t* x;  // [NB][cols]
  float* y;           // [NB][rows] (epilogue 0)
  // optional fused neighbours of the linear layer
  const uint16_t* gain;  // non-null: x is first RMS-normalised with this gain (rounded to bf16)
  float eps;
  int epi;               // 0: y = W x;  1: h = bf16(h + bf16(W x));  2: act[i] = swiglu(rows 2i, 2i+1)
  uint16_t* out16;       // h [NB][rows] (epilogue 1) or act [NB][rows/2] (epilogue 2)
  // shared-exponent form only: one exponent byte per bitmap word, ew bytes per row
  const uint8_t* sexp;
  int ew;
};

template <int FW>
struct Window {
  uint32_t m;
  uint32_t sh;
  uint32_t e;  // shared exponent of the lane's word (shared-exponent form)
  uint32_t d[FW + 1];
};

struct Cursor {  // walks the (row, chunk) items of one wave in order
  int row, chunk;
  // pair == 0: rows gw, gw + nwaves, ...; pair == 1: row pairs (2u, 2u+1) for u = gw, gw + nwaves, ...
  __device__ __forceinline__ void advance(int nchunk, int nwaves, int pair) {
    if (++chunk == nchunk) {
      chunk = 0;
      row += pair ? ((row & 1) ? 2 * nwaves - 1 : 1) : nwaves;
    }
  }
};

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kRawBufferFlags = 0x00020000;  // word 3 of a raw (unstructured, 32-bit data) buffer descriptor

constexpr int kGemvThreads = 1024;  // 16 waves share one staged copy of x
constexpr int kGemvWaves = kGemvThreads / 64;

// x in LDS: fp32 for one column; bf16 bit patterns (XH) for a batch, whose gathers of NB
// values per kept weight would otherwise saturate the LDS (measured 2.4x slower at NB = 4).
// The staged values are bf16-representable either way; XH costs one shift per use.
// Layout: per chunk of 64 bitmap words a block [1 + 32][64 lanes][NB]; row 0 holds zeros, row
// 1 + k the values of column k of every lane's word.  A lane only ever reads entries of its own
// 4-byte column of the block, so the gathers of a wave never meet in a bank whatever positions
// the lanes are at (with one 33-entry segment per lane they collided at ~3.8 extra cycles per
// gather, which made the LDS a co-limit of the kernel).
constexpr int kXRows = 33;
template <int NB>
__device__ __forceinline__ int x_index(int col) {  // index of x[col][0] in the staged layout
  const int w = col >> 5;
  return (((w >> 6) * kXRows + 1 + (col & 31)) * 64 + (w & 63)) * NB;
}
template <bool XH>
struct XStage {
  using type = float;
  static __device__ __forceinline__ float put(float v) { return v; }
  static __device__ __forceinline__ float get(float v) { return v; }
};
template <>
struct XStage<true> {
  using type = uint16_t;
  static __device__ __forceinline__ uint16_t put(float v) { return (uint16_t)(__float_as_uint(v) >> 16); }
  static __device__ __forceinline__ float get(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
};

// MX = false: fields of 16-T bits, the leading bits of the bf16 word.  MX = true: fields of
// 9-T bits (sign, 8-T leading magnitude bits) and one shared exponent per bitmap word: the
// products of a word are summed unscaled and multiplied once by 2^(E + T - 134).
template <int T, int NB, bool MX>
__global__ __launch_bounds__(kGemvThreads) void gemv_draft_kernel(GemvArgs a) {
  constexpr int FW = MX ? 9 - T : 16 - T;
  constexpr bool XH = NB > 1;
  using XS = XStage<XH>;
  using XT = typename XS::type;
  extern __shared__ uint8_t xs_raw[];
  XT* xs = reinterpret_cast<XT*>(xs_raw);
  const int tid = threadIdx.x;
  const int nchunk = (a.bw + 63) >> 6;
  const int nseg = nchunk * 64;
  const int lane = tid & 63;
  // wave-uniform values are made scalar explicitly so the row/chunk bookkeeping runs on the SALU
  // rows (row pairs) are dealt round-robin to the waves, numbered so that consecutive units go
  // to consecutive workgroups: every workgroup, and every SIMD inside it, gets the same count
  // within one
  const int gw = __builtin_amdgcn_readfirstlane(tid >> 6) * gridDim.x + blockIdx.x;
  const int nwaves = a.nwaves;
  const int pair = a.epi == 2;
  const int row_first = pair ? 2 * gw : gw;
  const bool idle = row_first >= a.rows;  // still helps staging x

  // bitmap words come through a buffer descriptor of the row's words: a word index past the row's
  // end, or a row past the matrix (no records), reads as 0 without a branch
  auto load_bm = [&](const Cursor& c) -> uint32_t {
    const int row = c.row < a.rows ? c.row : 0;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.bitmap + (size_t)row * a.bw), 0, c.row < a.rows ? a.bw * 4 : 0, kRawBufferFlags);
    return __builtin_amdgcn_raw_buffer_load_b32(rs, (c.chunk * 64 + lane) * 4, 0, 0);
  };
  uint32_t rowprefix = 0;  // kept values of the row before the chunk being issued
  auto issue = [&](const Cursor& c, uint32_t m, Window<FW>& w) {
    w.m = m;
    int cnt = __popc(m);
    int incl = wave_incl_scan(cnt);
    int total = __builtin_amdgcn_readlane(incl, 63);
    uint32_t p = rowprefix + (uint32_t)(incl - cnt);
    rowprefix = (c.chunk == nchunk - 1) ? 0u : rowprefix + (uint32_t)total;
    uint32_t bit = __umul24(p, FW);  // p < 2^20: one full-rate multiply
    w.sh = bit & 31u;
    int row = c.row < a.rows ? c.row : row_first;  // past the end: any valid row, its bitmap word is 0
    // The window is read through a buffer descriptor of the row's own part of the stream: words past
    // the row's end read as 0 (range check per word), so a lane that has run out of kept values
    // forms its leftover products from fields of this row or from zeros, never from misaligned bits
    // of the next row (which could look like Inf or NaN and turn 0 * f into NaN).
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.spec + (size_t)row * a.sw), 0, a.sw * 4, kRawBufferFlags);
    const int voff = (int)(bit >> 5) * 4;
#pragma unroll
    for (int j = 0; j + 4 <= FW + 1; j += 4) {
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, voff + 4 * j, 0, 0);
      w.d[j] = v.x; w.d[j + 1] = v.y; w.d[j + 2] = v.z; w.d[j + 3] = v.w;
    }
#pragma unroll
    for (int j = (FW + 1) & ~3; j <= FW; ++j) w.d[j] = __builtin_amdgcn_raw_buffer_load_b32(rs, voff + 4 * j, 0, 0);
    if constexpr (MX) {
      const int wi = c.chunk * 64 + lane;
      w.e = wi < a.bw ? a.sexp[(size_t)row * a.ew + wi] : 0u;
    }
  };

  float acc[NB], gate[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) acc[b] = gate[b] = 0.f;

  auto compute = [&](const Cursor& c, const Window<FW>& w) {
    uint32_t win[FW];
#pragma unroll
    for (int j = 0; j < FW; ++j) win[j] = __builtin_amdgcn_alignbit(w.d[j + 1], w.d[j], w.sh);
    uint32_t m = w.m;
    const XT* xb = xs + ((c.chunk * kXRows + 1) * 64 + lane) * NB;
    float accw[NB];  // shared-exponent form: unscaled sum of the lane's word
#pragma unroll
    for (int b = 0; b < NB; ++b) accw[b] = 0.f;
    auto step = [&](auto I) {
      constexpr int i = decltype(I)::value;
      int pos = lowest_bit(m);
      m &= m - 1u;
      const uint32_t top = field_top<FW, i>(win);
      const XT* xp = xb + pos * (64 * NB);
      if constexpr (MX) {
        // sign at bit 31, magnitude below it; a lane past its last field reads neighbouring
        // bits, always a finite number, and multiplies it by the zero entry of the segment
        const float mag = (float)__builtin_amdgcn_ubfe(top, 32 - FW, FW - 1);
        const float f = __uint_as_float((top & 0x80000000u) | __float_as_uint(mag));
#pragma unroll
        for (int b = 0; b < NB; ++b) accw[b] = fmaf(f, XS::get(xp[b]), accw[b]);
      } else {
        const float f = __uint_as_float(top);
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = fmaf(f, XS::get(xp[b]), acc[b]);
      }
    };
    // the first 16 set bits unconditionally, then pairs until every lane has run out
    static_for<0, 16>(step);
    auto tail = [&](auto self, auto I) -> void {
      constexpr int i = decltype(I)::value;
      if constexpr (i < 32) {
        if (__builtin_amdgcn_ballot_w64(m != 0u)) {
          step(std::integral_constant<int, i>{});
          step(std::integral_constant<int, i + 1>{});
          self(self, std::integral_constant<int, i + 2>{});
        }
      }
    };
    tail(tail, std::integral_constant<int, 16>{});
    if constexpr (MX) {
      const float scale = ldexpf(1.0f, (int)w.e + T - 134);
#pragma unroll
      for (int b = 0; b < NB; ++b) acc[b] = fmaf(accw[b], scale, acc[b]);
    }
    if (c.chunk == nchunk - 1) {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        float s = wave_sum(acc[b]);
        acc[b] = 0.f;
        if (a.epi == 0) {
          if (lane == 0) a.y[(size_t)b * a.rows + c.row] = s;
        } else if (a.epi == 1) {
          uint16_t* hp = a.out16 + (size_t)b * a.rows + c.row;
          if (lane == 0) *hp = f32_to_bf16(bf16_to_f32(*hp) + round_bf16(s));
        } else {
          if (c.row & 1) {  // up row: the gate row came just before
            const float g = round_bf16(gate[b]), u = round_bf16(s);
            if (lane == 0) a.out16[(size_t)b * (a.rows >> 1) + (c.row >> 1)] = f32_to_bf16(g / (1.0f + expf(-g)) * u);
          } else {
            gate[b] = s;
          }
        }
      }
    }
  };

  // ---- x is staged in blocks [chunk][1 + 32][64][NB]; row 0 of a block is 0.0.
  // Fast path (cols a multiple of 8, at most 2 pieces of 8 per thread): x and the norm gain are
  // read once with 16-byte loads, requested before anything else so they travel together with
  // the first bitmap words, and stay in registers between the norm reduction and the LDS writes.
  const int npiece = (nseg * 32) >> 3;  // pieces of 8 columns, including the zero tail
  const bool fast = (a.cols & 7) == 0 && npiece <= 2 * kGemvThreads &&
                    ((reinterpret_cast<uintptr_t>(a.x) | reinterpret_cast<uintptr_t>(a.gain)) & 15) == 0;
  uint4 raw[2][NB], gv[2];
  auto stage_load = [&]() {
    if (!fast) return;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int col = (tid + k * kGemvThreads) * 8;
      gv[k] = make_uint4(0, 0, 0, 0);
      if (a.gain && col < a.cols) gv[k] = *reinterpret_cast<const uint4*>(a.gain + col);
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        raw[k][b] = make_uint4(0, 0, 0, 0);
        if (col < a.cols) raw[k][b] = *reinterpret_cast<const uint4*>(a.x + (size_t)b * a.cols + col);
      }
    }
  };
  auto stage_x = [&]() {
    for (int sgi = tid; sgi < nseg; sgi += kGemvThreads) {
#pragma unroll
      for (int b = 0; b < NB; ++b) xs[(((sgi >> 6) * kXRows) * 64 + (sgi & 63)) * NB + b] = XS::put(0.f);
    }
    float rn[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) rn[b] = 1.f;
    __shared__ float red[NB][kGemvWaves];
    auto finish_norm = [&](const float (&ss)[NB]) {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        float t = wave_sum(ss[b]);
        if (lane == 0) red[b][tid >> 6] = t;
      }
      __syncthreads();
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < kGemvWaves; ++w) t += red[b][w];
        rn[b] = 1.0f / sqrtf(t / (float)a.cols + a.eps);
      }
    };
    if (fast) {
      if (a.gain) {
        float ss[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          ss[b] = 0.f;
#pragma unroll
          for (int k = 0; k < 2; ++k) {
            const uint32_t wd[4] = {raw[k][b].x, raw[k][b].y, raw[k][b].z, raw[k][b].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float lo = __uint_as_float(wd[e] << 16), hi = __uint_as_float(wd[e] & 0xFFFF0000u);
              ss[b] += lo * lo;
              ss[b] += hi * hi;
            }
          }
        }
        finish_norm(ss);
      }
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int piece = tid + k * kGemvThreads;
        const int col = piece * 8;
        if (piece < npiece) {
          const uint32_t gw4[4] = {gv[k].x, gv[k].y, gv[k].z, gv[k].w};
          XT* dst = xs + x_index<NB>(col);  // the 8 columns of a piece lie in one word: 64 * NB apart
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            const uint32_t wd[4] = {raw[k][b].x, raw[k][b].y, raw[k][b].z, raw[k][b].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float lo = __uint_as_float(wd[e] << 16), hi = __uint_as_float(wd[e] & 0xFFFF0000u);
              if (a.gain) {
                lo = round_bf16(lo * rn[b] * __uint_as_float(gw4[e] << 16));
                hi = round_bf16(hi * rn[b] * __uint_as_float(gw4[e] & 0xFFFF0000u));
              }
              dst[(2 * e) * 64 * NB + b] = XS::put(lo);
              dst[(2 * e + 1) * 64 * NB + b] = XS::put(hi);
            }
          }
        }
      }
    } else {
      if (a.gain) {
        float ss[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          ss[b] = 0.f;
          for (int c = tid; c < a.cols; c += kGemvThreads) {
            float v = bf16_to_f32(a.x[(size_t)b * a.cols + c]);
            ss[b] += v * v;
          }
        }
        finish_norm(ss);
      }
      for (int col = tid; col < nseg * 32; col += kGemvThreads) {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          float v = 0.f;
          if (col < a.cols) {
            v = bf16_to_f32(a.x[(size_t)b * a.cols + col]);
            if (a.gain) v = round_bf16(v * rn[b] * bf16_to_f32(a.gain[col]));
          }
          xs[x_index<NB>(col) + b] = XS::put(v);
        }
      }
    }
    __syncthreads();
  };
  Cursor cb{row_first, 0}, ci{row_first, 0}, cc{row_first, 0};
  Window<FW> w0, w1;
  stage_load();
  if (idle) {
    stage_x();
    return;
  }
  uint32_t m0 = load_bm(cb); cb.advance(nchunk, nwaves, pair);
  uint32_t m1 = load_bm(cb); cb.advance(nchunk, nwaves, pair);
  issue(ci, m0, w0); ci.advance(nchunk, nwaves, pair);
  stage_x();  // overlaps the first bitmap and window loads
  while (true) {
    uint32_t m2 = load_bm(cb); cb.advance(nchunk, nwaves, pair);
    issue(ci, m1, w1); ci.advance(nchunk, nwaves, pair);
    compute(cc, w0); cc.advance(nchunk, nwaves, pair);
    if (cc.row >= a.rows) break;
    m1 = load_bm(cb); cb.advance(nchunk, nwaves, pair);
    issue(ci, m2, w0); ci.advance(nchunk, nwaves, pair);
    compute(cc, w1); cc.advance(nchunk, nwaves, pair);
    if (cc.row >= a.rows) break;
  }
}

// LDS allowance of the instantiation, then the launch
template <int T, int NB, bool MX>
static int launch_gemv_instance(cas_ctx* ctx, const GemvArgs& a, int grid, size_t lds) {
  static LdsLimit lim;
  const int rc = allow_lds(ctx, (const void*)gemv_draft_kernel<T, NB, MX>, lds, lim);
  if (rc != CAS_OK) return rc;
  hipLaunchKernelGGL((gemv_draft_kernel<T, NB, MX>), dim3(grid), dim3(kGemvThreads), lds, ctx->stream, a);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

// LDS bytes of the staged x
static inline size_t gemv_lds_bytes(int bw, int batch) {
  return (batch > 1 ? sizeof(uint16_t) : sizeof(float)) * (size_t)((bw + 63) / 64 * 64) * 33 * batch;
}

// one or two workgroups per CU (two fill its 32 wave slots), whichever leaves the most loaded
// CU with fewer units (rows, or gate/up row pairs); all of them are resident at once
static inline int gemv_grid(const cas_ctx* ctx, int64_t units) {
  int64_t best_load = 0;
  int grid = 1;
  for (int g = 1; g <= 2; ++g) {
    const int64_t wgs = std::min<int64_t>((int64_t)ctx->num_cu * g, units);
    const int64_t load = (units + wgs - 1) / wgs * g;
    if (g == 1 || load < best_load) { best_load = load; grid = (int)wgs; }
  }
  return grid;
}

}  // namespace cas
