// Verification GEMM for 9 to 32 columns on the raw form: instantiates the wide forms of the kernel
// (see gemm_verify_kernel.inl) in a translation unit of their own.
#include "gemm_verify_kernel.inl"

namespace cas {

int launch_gemm_verify_wide(cas_ctx* ctx, const VerifyArgs& a, int t) { return verify_wide<false>(ctx, a, t); }

}  // namespace cas
