// Weight formatting (selection + truncation + split + pack) and dense reconstruction.
//
// Encode follows Sec. 4.2 of the paper: per output row the K best scores |W_ij| * a_j are the
// speculation group, their low t mantissa bits and all other values are the verification
// group (Sec. 4.1).  One workgroup formats one row: a 4-pass radix select finds the K-th
// largest score, equal scores are granted in ascending column order, fields are gathered in
// LDS bit streams and flushed with coalesced stores.
#include "cas_device.hpp"
#include "cas_internal.hpp"

namespace cas {

struct CodecArgs {
  int64_t rows, cols, ld;
  int K, t, bw, sw, lw, pw;
  uint32_t* bitmap;
  uint32_t* spec;
  uint32_t* lo;
  uint32_t* pruned;
};

__device__ __forceinline__ uint32_t score_of(uint16_t w, const float* __restrict__ act, int64_t j) {
  uint32_t mag = w & 0x7FFFu;
  if (!act) return mag;
  float s = __fmul_rn(__uint_as_float(mag << 16), act[j]);
  uint32_t b = __float_as_uint(s);
  return (s != s) ? 0x7FFFFFFFu : b;
}

__device__ __forceinline__ void put_field(uint32_t* s, uint32_t bit, uint32_t v, int width) {
  uint32_t w = bit >> 5, sh = bit & 31;
  atomicOr(&s[w], v << sh);
  if (sh + width > 32) atomicOr(&s[w + 1], v >> (32 - sh));
}

__global__ __launch_bounds__(256) void encode_rows_kernel(const uint16_t* __restrict__ W,
                                                          const float* __restrict__ act, CodecArgs a) {
  extern __shared__ uint32_t smem[];
  uint32_t* st_spec = smem;
  uint32_t* st_lo = st_spec + a.sw;
  uint32_t* st_pr = st_lo + a.lw;
  uint32_t* hist = st_pr + a.pw;   // 256
  uint32_t* eqc = hist + 256;      // bw
  uint32_t* gtc = eqc + a.bw;      // bw
  __shared__ uint32_t sh_prefix, sh_kk;

  const int tid = threadIdx.x;
  const int cols = (int)a.cols;
  if (blockIdx.x == 0 && tid < 64) {  // the slack kernels may over-read must hold finite values
    a.spec[a.rows * a.sw + tid] = 0;
    a.lo[a.rows * a.lw + tid] = 0;
    a.pruned[a.rows * a.pw + tid] = 0;
  }
  for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
    const uint16_t* wr = W + row * a.ld;
    for (int i = tid; i < a.sw + a.lw + a.pw; i += 256) smem[i] = 0;
    // ---- K-th largest score by radix select, most significant byte first
    uint32_t T = 0xFFFFFFFFu, need = 0;
    if (a.K > 0) {
      if (tid == 0) { sh_prefix = 0; sh_kk = (uint32_t)a.K; }
      for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh_prefix;
        const uint32_t himask = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
        for (int j = tid; j < cols; j += 256) {
          uint32_t s = score_of(wr[j], act, j);
          if ((s & himask) == prefix) atomicAdd(&hist[(s >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
          uint32_t kk = sh_kk, cum = 0;
          int b = 255;
          for (; b > 0; --b) {
            if (cum + hist[b] >= kk) break;
            cum += hist[b];
          }
          sh_kk = kk - cum;
          sh_prefix = prefix | ((uint32_t)b << shift);
        }
        __syncthreads();
      }
      T = sh_prefix;
      need = sh_kk;
    }
    // ---- per 32-column word: how many scores above / equal to the threshold
    for (int wd = tid; wd < a.bw; wd += 256) {
      uint32_t e = 0, g = 0;
      for (int c = 0; c < 32; ++c) {
        int j = wd * 32 + c;
        if (j < cols) {
          uint32_t s = score_of(wr[j], act, j);
          e += (s == T);
          g += (s > T);
        }
      }
      eqc[wd] = e;
      gtc[wd] = g;
    }
    __syncthreads();
    if (tid == 0) {  // exclusive prefix over the words, in column order
      uint32_t e = 0, g = 0;
      for (int wd = 0; wd < a.bw; ++wd) {
        uint32_t te = eqc[wd], tg = gtc[wd];
        eqc[wd] = e;
        gtc[wd] = g;
        e += te;
        g += tg;
      }
    }
    __syncthreads();
    // ---- mark, split and pack
    const int fw = 16 - a.t;
    const uint32_t lomask = (1u << a.t) - 1u;
    for (int wd = tid; wd < a.bw; wd += 256) {
      uint32_t eq_run = eqc[wd];
      uint32_t p = gtc[wd] + min(eq_run, need);  // kept values before this word
      uint32_t u = (uint32_t)wd * 32u - p;       // pruned values before this word
      uint32_t m = 0;
      for (int c = 0; c < 32; ++c) {
        int j = wd * 32 + c;
        if (j >= cols) break;
        uint16_t w = wr[j];
        uint32_t s = score_of(w, act, j);
        bool kept = s > T;
        if (s == T) {
          kept = eq_run < need;
          ++eq_run;
        }
        if (kept) {
          m |= 1u << c;
          put_field(st_spec, p * fw, (uint32_t)w >> a.t, fw);
          if (a.t) put_field(st_lo, p * a.t, (uint32_t)w & lomask, a.t);
          ++p;
        } else {
          put_field(st_pr, u * 16, w, 16);
          ++u;
        }
      }
      a.bitmap[row * a.bw + wd] = m;
    }
    __syncthreads();
    for (int i = tid; i < a.sw; i += 256) a.spec[row * a.sw + i] = st_spec[i];
    for (int i = tid; i < a.lw; i += 256) a.lo[row * a.lw + i] = st_lo[i];
    for (int i = tid; i < a.pw; i += 256) a.pruned[row * a.pw + i] = st_pr[i];
    __syncthreads();
  }
}

// Dense reconstruction of one row per workgroup; full == 0 gives the zero-padded draft view.
__global__ __launch_bounds__(256) void decode_rows_kernel(CodecArgs a, uint16_t* __restrict__ out, int full) {
  extern __shared__ uint32_t smem[];
  uint32_t* pre = smem;  // bw
  const int tid = threadIdx.x;
  const int cols = (int)a.cols;
  const int fw = 16 - a.t;
  for (int64_t row = blockIdx.x; row < a.rows; row += gridDim.x) {
    const uint32_t* bm = a.bitmap + row * a.bw;
    for (int wd = tid; wd < a.bw; wd += 256) pre[wd] = __popc(bm[wd]);
    __syncthreads();
    if (tid == 0) {
      uint32_t s = 0;
      for (int wd = 0; wd < a.bw; ++wd) {
        uint32_t t = pre[wd];
        pre[wd] = s;
        s += t;
      }
    }
    __syncthreads();
    const uint32_t* sp = a.spec + row * a.sw;
    const uint32_t* lo = a.lo + row * a.lw;
    const uint32_t* pr = a.pruned + row * a.pw;
    for (int wd = tid; wd < a.bw; wd += 256) {
      uint32_t m = bm[wd];
      uint32_t p = pre[wd], u = (uint32_t)wd * 32u - p;
      for (int c = 0; c < 32; ++c) {
        int j = wd * 32 + c;
        if (j >= cols) break;
        uint32_t v;
        if ((m >> c) & 1u) {
          v = read_field(sp, p * fw, fw) << a.t;
          if (full && a.t) v |= read_field(lo, p * a.t, a.t);
          ++p;
        } else {
          v = full ? read_field(pr, u * 16, 16) : 0u;
          ++u;
        }
        out[row * a.ld + j] = (uint16_t)v;
      }
    }
    __syncthreads();
  }
}

static CodecArgs make_args(const cas_wdesc& d, const void* spec, const void* verif, int64_t ld) {
  CodecArgs a;
  a.rows = d.rows; a.cols = d.cols; a.ld = ld;
  a.K = d.K; a.t = d.t; a.bw = d.bw; a.sw = d.sw; a.lw = d.lw; a.pw = d.pw;
  char* s = (char*)spec;
  char* v = (char*)verif;
  a.bitmap = (uint32_t*)(s + d.off_bitmap);
  a.spec = (uint32_t*)(s + d.off_spec);
  a.lo = v ? (uint32_t*)(v + d.off_lo) : nullptr;
  a.pruned = v ? (uint32_t*)(v + d.off_pruned) : nullptr;
  return a;
}

int launch_encode_weight(cas_ctx* ctx, const uint16_t* W, int64_t ld, const float* act, const cas_wdesc& d,
                         void* spec, void* verif) {
  CodecArgs a = make_args(d, spec, verif, ld);
  size_t lds = sizeof(uint32_t) * ((size_t)d.sw + d.lw + d.pw + 256 + 2 * (size_t)d.bw);
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  static LdsLimit lim;
  const int rc = allow_lds(ctx, (const void*)encode_rows_kernel, lds, lim);
  if (rc != CAS_OK) return rc;
  int grid = (int)std::min<int64_t>(d.rows, (int64_t)ctx->num_cu * 8);
  if (grid < 1) return CAS_OK;
  hipLaunchKernelGGL(encode_rows_kernel, dim3(grid), dim3(256), lds, ctx->stream, W, act, a);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

int launch_decode_weight(cas_ctx* ctx, const cas_wdesc& d, const void* spec, const void* verif, uint16_t* out,
                         int64_t ld) {
  CodecArgs a = make_args(d, spec, verif, ld);
  size_t lds = sizeof(uint32_t) * (size_t)d.bw;
  int grid = (int)std::min<int64_t>(d.rows, (int64_t)ctx->num_cu * 8);
  if (grid < 1) return CAS_OK;
  hipLaunchKernelGGL(decode_rows_kernel, dim3(grid), dim3(256), lds, ctx->stream, a, out, verif ? 1 : 0);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

}  // namespace cas
