// Partial attention kernel over a cache in the shared-exponent form (Sec. 4.2, the MX approach):
// the kernel template of attention.hip with the kept walk that rebuilds a bf16 word from sign,
// magnitude and the exponent of the vector's 32-channel block; the exact form.  A translation
// unit of its own so that the build compiles it beside the others.
#include "attention_kernel.inl"

namespace cas {
template int launch_mt<1, true, true>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<2, true, true>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<3, true, true>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<4, true, true>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<5, true, true>(cas_ctx*, const AttnBatch&, dim3);
}  // namespace cas
