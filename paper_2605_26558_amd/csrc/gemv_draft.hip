// Draft GEMV: y = Wdraft x, reading only the speculation data (bitmap + spec stream) and
// decoding it inside the kernel (Sec. 4.1 draft inference: zero padding of pruned positions
// and dropped mantissa bits).
//
// Mapping.  One wave walks one output row at a time in chunks of 64 bitmap words (2048
// columns): lane l owns word l of the chunk, i.e. 32 consecutive columns.  A DPP prefix sum of
// the popcounts gives each lane the index of its first kept value, so its fields are one
// contiguous run of the row's spec stream; neighbouring lanes read neighbouring runs.  The
// lane loads a window of 16-t+1 words at its run, aligns it with funnel shifts, and then
// walks the set bits of its word: field i of the window belongs to the i-th set bit.  Placing
// a field at the top of a 32-bit register yields the fp32 value of the zero-padded bf16.
// x sits in LDS as fp32 in segments of 1+32 entries per bitmap word; entry 0 of a segment is
// 0.0, so a lane that has run out of set bits (bit position -1) multiplies by zero.
// The (row, chunk) items of a wave run through a three-stage software pipeline: bitmap word of
// item q+2, prefix + window loads of item q+1, arithmetic of item q.
#include "gemv_draft_kernel.inl"

namespace cas {

template <int T>
static int launch_t(cas_ctx* ctx, const GemvArgs& a, int batch, int grid, size_t lds) {
  switch (batch) {
    case 1: return launch_gemv_instance<T, 1, false>(ctx, a, grid, lds);
    case 2: return launch_gemv_instance<T, 2, false>(ctx, a, grid, lds);
    case 3: return launch_gemv_instance<T, 3, false>(ctx, a, grid, lds);
    case 4: return launch_gemv_instance<T, 4, false>(ctx, a, grid, lds);
    default: return CAS_EINVAL;
  }
}

int launch_gemv_draft(cas_ctx* ctx, const cas_wdesc& d, const void* spec, const uint16_t* x, int batch, float* y) {
  return launch_gemv_draft_fused(ctx, d, spec, x, batch, y, nullptr, 0.f, 0, nullptr);
}

int launch_gemv_draft_fused(cas_ctx* ctx, const cas_wdesc& d, const void* spec, const uint16_t* x, int batch,
                            float* y, const uint16_t* gain, float eps, int epi, uint16_t* out16) {
  if (d.rows <= 0) return CAS_OK;
  if (epi == 2 && (d.rows & 1)) return CAS_EINVAL;
  GemvArgs a{};
  a.gain = gain; a.eps = eps; a.epi = epi; a.out16 = out16;
  a.rows = (int)d.rows; a.cols = (int)d.cols; a.bw = d.bw; a.sw = d.sw;
  a.bitmap = (const uint32_t*)((const char*)spec + d.off_bitmap);
  a.spec = (const uint32_t*)((const char*)spec + d.off_spec);
  a.x = x; a.y = y;
  // x: fp32 for one column, bf16 for a batch (see XStage)
  const size_t lds = gemv_lds_bytes(d.bw, batch);
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  const int grid = gemv_grid(ctx, epi == 2 ? d.rows / 2 : d.rows);  // a gate/up row pair stays in one wave
  a.nwaves = grid * kGemvWaves;
  ProfScope prof(ctx, PROF_GEMV_DRAFT, 4.0 * (double)d.rows * (d.bw + d.sw));
#define CAS_T(TV) case TV: return launch_t<TV>(ctx, a, batch, grid, lds);
  switch (d.t) {
    CAS_T(0) CAS_T(1) CAS_T(2) CAS_T(3) CAS_T(4) CAS_T(5) CAS_T(6) CAS_T(7)
  }
#undef CAS_T
  return CAS_EINVAL;
}

}  // namespace cas
