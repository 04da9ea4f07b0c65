// Draft form of the partial attention kernel (K and V rebuilt from the speculation data alone,
// Sec. 4.1); compiled apart from the exact form to halve the build time.
#include "attention_kernel.inl"

namespace cas {
template int launch_mt<1, false, false>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<2, false, false>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<3, false, false>(cas_ctx*, const AttnBatch&, dim3);
}  // namespace cas
