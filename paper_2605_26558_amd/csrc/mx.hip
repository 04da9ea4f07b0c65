// Speculation data with shared exponents (Sec. 4.2 "Exponent Compression", the MX approach;
// decoder #N of Sec. 5.1): re-coding of an encoded matrix, reconstruction, and the draft GEMV
// on the shared-exponent form (the kernel template of the raw form with a different field
// decode: integer magnitude -> float, one scale per bitmap word).
#include "gemv_draft_kernel.inl"

namespace cas {

struct MxArgs {
  int rows, cols, K, t, bw, sw, lw, pw, fw, ew;
  // raw form (input of the re-coding)
  const uint32_t* bitmap;
  const uint32_t* spec;
  const uint32_t* lo;
  // shared-exponent form
  uint32_t* m_bitmap;
  uint8_t* m_sexp;
  uint32_t* m_field;
  uint32_t* m_lo;
  const uint32_t* m_pruned;
};

// OR a field of `width` bits into a zeroed little-endian bit stream
__device__ __forceinline__ void or_field(uint32_t* row, uint32_t index, int width, uint32_t v) {
  const uint32_t bit = index * (uint32_t)width, sh = bit & 31u;
  atomicOr(&row[bit >> 5], v << sh);
  if (sh + width > 32) atomicOr(&row[(bit >> 5) + 1], v >> (32u - sh));
}

// ---- re-coding: one wave per row, one bitmap word (= one block) per lane ---------------------
// field and lo regions are zero before this kernel; bits are OR-ed in.
__global__ __launch_bounds__(256) void mx_encode_kernel(MxArgs a) {
  const int lane = threadIdx.x & 63, gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
  const int HW = 16 - a.t, FB = 9 - a.t;
  for (int row = gw; row < a.rows; row += nw) {
    const uint32_t* sp_row = a.spec + (size_t)row * a.sw;
    const uint32_t* lo_row = a.lo + (size_t)row * a.lw;
    uint32_t* f_row = a.m_field + (size_t)row * a.fw;
    uint32_t* l_row = a.m_lo + (size_t)row * a.lw;
    int base = 0;
    for (int w0 = 0; w0 < a.bw; w0 += 64) {
      const int w = w0 + lane;
      const uint32_t m = w < a.bw ? a.bitmap[(size_t)row * a.bw + w] : 0u;
      const int cnt = __popc(m);
      const int incl = wave_incl_scan(cnt);
      const int e0 = base + incl - cnt;
      base += __builtin_amdgcn_readlane(incl, 63);
      auto word_of = [&](int e) -> uint32_t {
        uint32_t v = read_field(sp_row, (uint32_t)e * HW, HW) << a.t;
        if (a.t > 0) v |= read_field(lo_row, (uint32_t)e * a.t, a.t);
        return v;
      };
      int E = 0;
      for (int j = 0; j < cnt; ++j) E = max(E, eff_exponent(word_of(e0 + j)));
      if (w < a.bw) {
        a.m_bitmap[(size_t)row * a.bw + w] = m;
        a.m_sexp[(size_t)row * a.ew + w] = (uint8_t)E;
      }
      for (int j = 0; j < cnt; ++j) {
        const uint32_t v = word_of(e0 + j);
        const int sh = E - eff_exponent(v);
        const uint32_t mag = sh < 8 ? significand(v) >> sh : 0u;
        or_field(f_row, (uint32_t)(e0 + j), FB, ((v >> 15) << (8 - a.t)) | (mag >> a.t));
        if (a.t > 0) or_field(l_row, (uint32_t)(e0 + j), a.t, mag & ((1u << a.t) - 1u));
      }
    }
  }
}

// ---- reconstruction (reference path): one wave per row ---------------------------------------
__global__ __launch_bounds__(256) void mx_decode_kernel(MxArgs a, uint16_t* __restrict__ out, int64_t ld, int full) {
  const int lane = threadIdx.x & 63, gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
  const int FB = 9 - a.t, HB = 8 - a.t;
  for (int row = gw; row < a.rows; row += nw) {
    const uint32_t* f_row = a.m_field + (size_t)row * a.fw;
    const uint32_t* l_row = a.m_lo + (size_t)row * a.lw;
    const uint32_t* pr_row = a.m_pruned + (size_t)row * a.pw;
    uint16_t* orow = out + (size_t)row * ld;
    int base = 0;
    for (int w0 = 0; w0 < a.bw; w0 += 64) {
      const int w = w0 + lane;
      uint32_t m = w < a.bw ? a.m_bitmap[(size_t)row * a.bw + w] : 0u;
      const int E = w < a.bw ? a.m_sexp[(size_t)row * a.ew + w] : 0;
      const int nvalid = a.cols - w * 32;
      const uint32_t valid = nvalid >= 32 ? 0xFFFFFFFFu : (nvalid <= 0 ? 0u : ((1u << nvalid) - 1u));
      uint32_t pm = ~m & valid;
      const int cnt = __popc(m);
      const int incl = wave_incl_scan(cnt);
      int e = base + incl - cnt;
      int u = w * 32 - e;  // pruned values before this word
      base += __builtin_amdgcn_readlane(incl, 63);
      while (m) {
        const int pos = lowest_bit(m);
        m &= m - 1u;
        const uint32_t f = read_field(f_row, (uint32_t)e * FB, FB);
        uint32_t mag = (f & ((1u << HB) - 1u)) << a.t;
        if (full && a.t > 0) mag |= read_field(l_row, (uint32_t)e * a.t, a.t);
        orow[w * 32 + pos] = (uint16_t)mx_word(f >> HB, E, mag);
        ++e;
      }
      while (pm) {
        const int pos = lowest_bit(pm);
        pm &= pm - 1u;
        orow[w * 32 + pos] = full ? (uint16_t)read_field(pr_row, (uint32_t)u * 16u, 16) : (uint16_t)0;
        ++u;
      }
    }
  }
}

static int64_t up256(int64_t v) { return (v + 255) / 256 * 256; }
constexpr int64_t kMxSlack = 256;

static void fill_layout(cas_mxdesc* x) {
  const cas_wdesc& d = x->base;
  x->fw = (int32_t)(((int64_t)d.K * (9 - d.t) + 31) / 32);
  x->ew = (d.bw + 3) / 4 * 4;
  x->off_bitmap = 0;
  x->off_sexp = up256(d.rows * d.bw * 4);
  x->off_field = up256(x->off_sexp + d.rows * (int64_t)x->ew);
  x->spec_bytes = up256(x->off_field + d.rows * (int64_t)x->fw * 4 + kMxSlack);
  x->off_lo = 0;
  x->off_pruned = up256(d.rows * (int64_t)d.lw * 4 + kMxSlack);
  x->verif_bytes = up256(x->off_pruned + d.rows * (int64_t)d.pw * 4 + kMxSlack);
}

static bool sane_base(const cas_wdesc& d) {
  return d.rows >= 0 && d.rows <= 0x7FFFFFFF && d.cols >= 1 && d.cols <= 0x7FFFFFFF && d.t >= 0 && d.t <= 7 &&
         d.K >= 0 && d.K <= d.cols && d.bw == (int32_t)((d.cols + 31) / 32) &&
         d.sw == (int32_t)(((int64_t)d.K * (16 - d.t) + 31) / 32) && d.lw == (int32_t)(((int64_t)d.K * d.t + 31) / 32) &&
         d.pw == (int32_t)(((d.cols - d.K) * 16 + 31) / 32);
}

static int check_mxdesc(const cas_mxdesc* x) {
  if (!x || !sane_base(x->base)) return CAS_EINVAL;
  cas_mxdesc chk = *x;
  fill_layout(&chk);
  if (chk.fw != x->fw || chk.ew != x->ew || chk.off_bitmap != x->off_bitmap || chk.off_sexp != x->off_sexp ||
      chk.off_field != x->off_field || chk.spec_bytes != x->spec_bytes || chk.off_lo != x->off_lo ||
      chk.off_pruned != x->off_pruned || chk.verif_bytes != x->verif_bytes)
    return CAS_EINVAL;
  return CAS_OK;
}

static MxArgs make_args(const cas_mxdesc& x, const void* spec, const void* verif, void* mspec, const void* mverif) {
  const cas_wdesc& d = x.base;
  MxArgs a{};
  a.rows = (int)d.rows; a.cols = (int)d.cols; a.K = d.K; a.t = d.t;
  a.bw = d.bw; a.sw = d.sw; a.lw = d.lw; a.pw = d.pw; a.fw = x.fw; a.ew = x.ew;
  if (spec) {
    a.bitmap = (const uint32_t*)((const char*)spec + d.off_bitmap);
    a.spec = (const uint32_t*)((const char*)spec + d.off_spec);
  }
  if (verif) a.lo = (const uint32_t*)((const char*)verif + d.off_lo);
  if (mspec) {
    char* b = (char*)mspec;
    a.m_bitmap = (uint32_t*)(b + x.off_bitmap);
    a.m_sexp = (uint8_t*)(b + x.off_sexp);
    a.m_field = (uint32_t*)(b + x.off_field);
  }
  if (mverif) {
    a.m_lo = (uint32_t*)((char*)const_cast<void*>(mverif) + x.off_lo);
    a.m_pruned = (const uint32_t*)((const char*)mverif + x.off_pruned);
  }
  return a;
}

static int row_grid(cas_ctx* ctx, int64_t rows) {
  return (int)std::max<int64_t>(1, std::min<int64_t>((rows + 3) / 4, (int64_t)ctx->num_cu * 8));
}

// Draft GEMV on the shared-exponent form with the epilogues of the raw form (one column).
int launch_gemv_draft_mx_fused(cas_ctx* ctx, const cas_mxdesc& mx, const void* d_mxspec, const uint16_t* d_x, float* d_y,
                               const uint16_t* gain, float eps, int epi, uint16_t* out16) {
  const cas_wdesc& d = mx.base;
  if (d.rows == 0) return CAS_OK;
  if (epi == 2 && (d.rows & 1)) return CAS_EINVAL;
  GemvArgs a{};
  a.gain = gain; a.eps = eps; a.epi = epi; a.out16 = out16;
  a.rows = (int)d.rows; a.cols = (int)d.cols; a.bw = d.bw; a.sw = mx.fw;
  a.bitmap = (const uint32_t*)((const char*)d_mxspec + mx.off_bitmap);
  a.spec = (const uint32_t*)((const char*)d_mxspec + mx.off_field);
  a.sexp = (const uint8_t*)d_mxspec + mx.off_sexp;
  a.ew = mx.ew;
  a.x = d_x; a.y = d_y;
  const size_t lds = gemv_lds_bytes(d.bw, 1);
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  const int grid = gemv_grid(ctx, epi == 2 ? d.rows / 2 : d.rows);  // a gate/up row pair stays in one wave
  a.nwaves = grid * kGemvWaves;
#define CAS_T(TV) case TV: return launch_gemv_instance<TV, 1, true>(ctx, a, grid, lds);
  switch (d.t) {
    CAS_T(0) CAS_T(1) CAS_T(2) CAS_T(3) CAS_T(4) CAS_T(5) CAS_T(6) CAS_T(7)
  }
#undef CAS_T
  return CAS_EINVAL;
}

bool mxdesc_ok(const cas_mxdesc* x) { return check_mxdesc(x) == CAS_OK; }

}  // namespace cas

using namespace cas;

extern "C" int cas_mx_plan(const cas_wdesc* desc, cas_mxdesc* out) {
  if (!desc || !out || !sane_base(*desc)) return CAS_EINVAL;
  *out = cas_mxdesc{};
  out->base = *desc;
  fill_layout(out);
  return CAS_OK;
}

extern "C" int cas_mx_encode(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_spec, const void* d_verif,
                             void* d_mxspec, void* d_mxverif) {
  if (!ctx || check_mxdesc(mx) != CAS_OK || !d_mxspec || !d_mxverif || !aligned256(d_mxspec) || !aligned256(d_mxverif))
    return CAS_EINVAL;
  const cas_wdesc& d = mx->base;
  CAS_HIP(ctx, hipMemsetAsync(d_mxspec, 0, (size_t)mx->spec_bytes, ctx->stream));
  CAS_HIP(ctx, hipMemsetAsync(d_mxverif, 0, (size_t)mx->verif_bytes, ctx->stream));
  if (d.rows == 0) return CAS_OK;
  if (!d_spec || !d_verif || !aligned256(d_spec) || !aligned256(d_verif)) return CAS_EINVAL;
  // the pruned stream is the raw one, word for word
  CAS_HIP(ctx, hipMemcpyAsync((char*)d_mxverif + mx->off_pruned, (const char*)d_verif + d.off_pruned,
                              (size_t)d.rows * d.pw * 4, hipMemcpyDeviceToDevice, ctx->stream));
  MxArgs a = make_args(*mx, d_spec, d_verif, d_mxspec, d_mxverif);
  hipLaunchKernelGGL(mx_encode_kernel, dim3(row_grid(ctx, a.rows)), dim3(256), 0, ctx->stream, a);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

extern "C" int cas_mx_decode(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_mxspec, const void* d_mxverif,
                             uint16_t* d_out, int64_t ld) {
  if (!ctx || check_mxdesc(mx) != CAS_OK || ld < mx->base.cols) return CAS_EINVAL;
  if (mx->base.rows == 0) return CAS_OK;
  if (!d_mxspec || !d_out || !aligned256(d_mxspec) || !aligned256(d_mxverif)) return CAS_EINVAL;
  MxArgs a = make_args(*mx, nullptr, nullptr, const_cast<void*>(d_mxspec), d_mxverif);
  hipLaunchKernelGGL(mx_decode_kernel, dim3(row_grid(ctx, a.rows)), dim3(256), 0, ctx->stream, a, d_out, ld,
                     d_mxverif ? 1 : 0);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

extern "C" int cas_gemv_draft_mx(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_mxspec, const uint16_t* d_x,
                                 float* d_y) {
  if (!ctx || check_mxdesc(mx) != CAS_OK) return CAS_EINVAL;
  const cas_wdesc& d = mx->base;
  if (d.rows == 0) return CAS_OK;
  if (!d_mxspec || !d_x || !d_y || !aligned256(d_mxspec)) return CAS_EINVAL;
  return launch_gemv_draft_mx_fused(ctx, *mx, d_mxspec, d_x, d_y, nullptr, 0.f, 0, nullptr);
}

extern "C" int cas_gemm_verify_mx(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_mxspec, const void* d_mxverif,
                                  const uint16_t* d_X, int ncols, float* d_Y) {
  if (!ctx || check_mxdesc(mx) != CAS_OK || ncols < 1 || ncols > 32) return CAS_EINVAL;
  if (mx->base.rows == 0) return CAS_OK;
  if (!d_mxspec || !d_mxverif || !d_X || !d_Y || !aligned256(d_mxspec) || !aligned256(d_mxverif)) return CAS_EINVAL;
  return launch_gemm_verify_mx_fused(ctx, *mx, d_mxspec, d_mxverif, d_X, ncols, d_Y, 0, nullptr);
}
