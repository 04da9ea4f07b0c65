// Verification GEMM: Y = W X with W rebuilt exactly from speculation + verification data
// inside the kernel (Sec. 4.1 target inference, Sec. 5.1 mantissa concatenation and bitmap
// de-sparsification) and X holding the k+1 columns of one verification pass (Sec. 2.2).
//
// Mapping.  A workgroup of four waves owns 16 output rows and walks the columns in slabs of
// 2048; wave w takes the w-th 512-column quarter of every slab.  Inside a quarter lane (r, j)
// owns bitmap words 4j..4j+3 of row r (128 consecutive columns), so its kept fields, dropped
// mantissa bits and pruned words are contiguous runs of the three streams.  For each of its
// four words the lane walks the set bits (kept: leading bits from spec, low bits from lo) and
// then the clear bits (pruned: verbatim word) and scatters the bf16 values into a 16 x 128
// tile in LDS.  The tile is then multiplied with the matching 128 rows of X by eight
// 16x16x16 bf16 MFMA operations, accumulating in fp32.  Every wave stages the X columns of
// its own part of the slab into its own LDS region, so waves never wait for each other inside
// the column loop.  Each output column uses the same
// sequence of operations whatever the number of columns is.  The four partial tiles of a
// workgroup are added in wave order through LDS.
#include "gemm_verify_kernel.inl"

namespace cas {

int launch_gemm_verify(cas_ctx* ctx, const cas_wdesc& d, const void* spec, const void* verif, const uint16_t* X,
                       int ncols, float* Y) {
  return launch_gemm_verify_fused(ctx, d, spec, verif, X, ncols, Y, 0, nullptr);
}

static int launch_verify_args(cas_ctx* ctx, const VerifyArgs& a, int t) {
  if (a.ncols > 8) return launch_gemm_verify_wide(ctx, a, t);
  return verify_narrow<false>(ctx, a, t);
}

int launch_gemm_verify_fused(cas_ctx* ctx, const cas_wdesc& d, const void* spec, const void* verif,
                             const uint16_t* X, int ncols, float* Y, int epi, uint16_t* out16) {
  if (d.rows <= 0) return CAS_OK;
  if (epi == 2 && (d.rows & 1)) return CAS_EINVAL;
  VerifyArgs a;
  a.epi = epi; a.out16 = out16;
  a.rows = (int)d.rows; a.cols = (int)d.cols; a.bw = d.bw; a.sw = d.sw; a.lw = d.lw; a.pw = d.pw;
  a.ncols = ncols;
  a.bitmap = (const uint32_t*)((const char*)spec + d.off_bitmap);
  a.spec = (const uint32_t*)((const char*)spec + d.off_spec);
  a.lo = (const uint32_t*)((const char*)verif + d.off_lo);
  a.pruned = (const uint32_t*)((const char*)verif + d.off_pruned);
  a.X = X; a.Y = Y; a.yld = (int)d.rows;
  a.sexp = nullptr; a.ew = 0;
  ProfScope prof(ctx, PROF_GEMM_VERIFY, 4.0 * (double)d.rows * (d.bw + d.sw + d.lw + d.pw));
  return launch_verify_args(ctx, a, d.t);
}

// The same product with the speculation data in the unary form (Sec. 4.2, the lossless
// configuration): blocks of rows are re-coded into the raw spec stream in the workspace and the
// kernel above runs on each block, so every output has the bits the raw form gives.
int launch_gemm_verify_unary_fused(cas_ctx* ctx, const cas_udesc& u, const void* uspec, const void* verif,
                                   const uint16_t* X, int ncols, float* Y, int epi, uint16_t* out16) {
  const cas_wdesc& d = u.base;
  if (d.rows <= 0) return CAS_OK;
  if (epi == 2 && (d.rows & 1)) return CAS_EINVAL;
  const size_t row_bytes = (size_t)d.sw * 4;
  // a block of rows: a multiple of 16 (whole row groups), as many as the workspace holds
  // (the kernel's windows read a little past the last field of a row: 256 bytes of slack behind the block)
  int64_t blk = row_bytes ? (ctx->ws_bytes > 256 ? (int64_t)((ctx->ws_bytes - 256) / row_bytes) : 0) : d.rows;
  blk = std::min<int64_t>(blk, d.rows);
  if (blk < d.rows) blk = blk / 16 * 16;
  if (blk < 1 || (d.sw > 0 && !ctx->d_ws)) return CAS_ENOMEM;
  ProfScope prof(ctx, PROF_GEMM_VERIFY, 4.0 * (double)d.rows * (d.bw + u.smw + d.lw + d.pw) + 4.0 * (double)u.ue_words);
  for (int64_t r0 = 0; r0 < d.rows; r0 += blk) {
    const int nr = (int)std::min<int64_t>(blk, d.rows - r0);
    int rc = launch_unary_expand(ctx, u, uspec, r0, nr, (uint32_t*)ctx->d_ws);
    if (rc != CAS_OK) return rc;
    VerifyArgs a;
    a.epi = epi;
    a.rows = nr; a.cols = (int)d.cols; a.bw = d.bw; a.sw = d.sw; a.lw = d.lw; a.pw = d.pw;
    a.ncols = ncols;
    a.bitmap = (const uint32_t*)((const char*)uspec + u.off_bitmap) + (size_t)r0 * d.bw;
    a.spec = (const uint32_t*)ctx->d_ws;
    a.lo = (const uint32_t*)((const char*)verif + d.off_lo) + (size_t)r0 * d.lw;
    a.pruned = (const uint32_t*)((const char*)verif + d.off_pruned) + (size_t)r0 * d.pw;
    a.X = X; a.yld = (int)d.rows;
    a.sexp = nullptr; a.ew = 0;
    a.Y = Y ? Y + r0 : nullptr;
    a.out16 = out16 ? out16 + (epi == 2 ? r0 / 2 : r0) : nullptr;
    rc = launch_verify_args(ctx, a, d.t);
    if (rc != CAS_OK) return rc;
  }
  return CAS_OK;
}

}  // namespace cas
