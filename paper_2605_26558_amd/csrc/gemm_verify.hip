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
  a.X = X; a.Y = Y;
  ProfScope prof(ctx, PROF_GEMM_VERIFY, 4.0 * (double)d.rows * (d.bw + d.sw + d.lw + d.pw));
  // One row group per workgroup.  Many row groups: four waves, each taking a quarter of every
  // slab (measured faster than 8-wave workgroups: fewer lanes wait at the slab barriers).  Few
  // row groups: eight waves so that every CU still gets several, sixteen when the rows are long
  // (each wave then has one decode step per slab and the serial chain per workgroup halves).
  // More than 8 columns: X is staged per decode step (see gemm_verify_wide.hip); up to 8 the
  // per-slab staging measured 5 % faster on the largest matrices.
  if (ncols > 8) return launch_gemm_verify_wide(ctx, a, d.t);
  const int groups = (int)((d.rows + 15) / 16);
  if (groups < kFewGroups && d.cols >= 4 * kSlabCols) return launch_gq<1, 16, 1, 1>(ctx, a, d.t);
  if (groups < kFewGroups) return launch_gq<1, 8, 2, 1>(ctx, a, d.t);
  return launch_gq<1, 4, 4, 1>(ctx, a, d.t);
}

}  // namespace cas
