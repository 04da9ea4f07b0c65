// Draft form of the partial attention kernel over a cache in the shared-exponent form: K and V from
// sign + leading magnitude bits and the block exponents alone (Sec. 4.1 draft inference on the
// Sec. 4.2 MX format).
#include "attention_kernel.inl"

namespace cas {
template int launch_mt<1, false, true>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<2, false, true>(cas_ctx*, const AttnBatch&, dim3);
template int launch_mt<3, false, true>(cas_ctx*, const AttnBatch&, dim3);
}  // namespace cas
