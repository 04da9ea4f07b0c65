// Verification GEMM on the shared-exponent form (Sec. 4.2, the MX approach, under Sec. 4.1 target
// inference): Y = W' X with W' the CONVERTED matrix.  The kernel of the raw form with one change
// in the kept walk: a field is sign + 8-t leading magnitude bits (t more from lo), and the walk
// writes the bf16 word of (-1)^sign * magnitude * 2^(E - 134), E being the exponent of the
// lane's bitmap word (one byte per word, read with the bitmaps).  Pruned values, tile, MFMA,
// reduction and epilogues are the raw form's; the forms are instantiated here, in a translation
// unit of their own.
#include "gemm_verify_kernel.inl"

namespace cas {

int launch_gemm_verify_mx_fused(cas_ctx* ctx, const cas_mxdesc& x, const void* mxspec, const void* mxverif,
                                const uint16_t* X, int ncols, float* Y, int epi, uint16_t* out16) {
  const cas_wdesc& d = x.base;
  if (d.rows <= 0) return CAS_OK;
  if (epi == 2 && (d.rows & 1)) return CAS_EINVAL;
  VerifyArgs a;
  a.epi = epi; a.out16 = out16;
  a.rows = (int)d.rows; a.cols = (int)d.cols; a.bw = d.bw; a.sw = x.fw; a.lw = d.lw; a.pw = d.pw;
  a.ncols = ncols;
  a.bitmap = (const uint32_t*)((const char*)mxspec + x.off_bitmap);
  a.spec = (const uint32_t*)((const char*)mxspec + x.off_field);
  a.sexp = (const uint8_t*)mxspec + x.off_sexp;
  a.ew = x.ew;
  a.lo = (const uint32_t*)((const char*)mxverif + x.off_lo);
  a.pruned = (const uint32_t*)((const char*)mxverif + x.off_pruned);
  a.X = X; a.Y = Y; a.yld = (int)d.rows;
  ProfScope prof(ctx, PROF_GEMM_VERIFY, 4.0 * (double)d.rows * (d.bw + x.fw + d.lw + d.pw) + (double)d.rows * x.ew);
  if (ncols > 8) return verify_wide<true>(ctx, a, d.t);
  return verify_narrow<true>(ctx, a, d.t);
}

}  // namespace cas
