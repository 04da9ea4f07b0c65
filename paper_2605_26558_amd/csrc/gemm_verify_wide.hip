// Verification GEMM for 9 to 32 columns (several sequences per pass, or long drafts): the same
// kernel as for few columns with X staged one decode step at a time, so that the LDS of a
// workgroup stays small enough for three of them per CU, and a second block of 16 output
// columns above 16.
#include "gemm_verify_kernel.inl"

namespace cas {

// The number of waves per row group depends on the matrix alone, never on the number of
// columns: it fixes the order in which a row's partial sums are added, and a column must get
// the same bits in every call.
template <int NB>
static int launch_nb(cas_ctx* ctx, const VerifyArgs& a, int t) {
  const int groups = (a.yld + 15) / 16;  // of the whole matrix, also when the launch covers a block of its rows
  if (groups < kFewGroups && a.cols >= 4 * kSlabCols) return launch_gq<1, 16, 1, NB>(ctx, a, t);
  if (groups < kFewGroups) return launch_gq<1, 8, 1, NB>(ctx, a, t);
  return launch_gq<1, 4, 1, NB>(ctx, a, t);
}

int launch_gemm_verify_wide(cas_ctx* ctx, const VerifyArgs& a, int t) {
  if (a.ncols <= 16) return launch_nb<1>(ctx, a, t);
  int rc = launch_nb<2>(ctx, a, t);
  if (rc != CAS_ENOTSUP) return rc;
  // sixteen waves per row group with more than 20 columns exceed the LDS: two launches of one
  // column block each (the weights of such a matrix are read twice)
  VerifyArgs lo = a, hi = a;
  lo.ncols = 16;
  hi.ncols = a.ncols - 16;
  hi.X = a.X + (size_t)16 * a.cols;
  if (a.Y) hi.Y = a.Y + (size_t)16 * a.yld;
  if (a.out16) hi.out16 = a.out16 + (size_t)16 * (a.epi == 2 ? a.yld >> 1 : a.yld);
  rc = launch_nb<1>(ctx, lo, t);
  if (rc != CAS_OK) return rc;
  return launch_nb<1>(ctx, hi, t);
}

}  // namespace cas
