// Dense bf16 GEMV y = W x on the uncompressed matrix: the BFloat16 baseline the paper normalises
// its speedups to (Sec. 7), written by hand so that the comparison does not rest on a vendor
// library.  HBM-bound by construction: 2 bytes per weight, two bit operations and one FMA per
// weight, far below the VALU budget.
//
// One wave per row at a time, rows dealt round-robin to all waves of the grid; a lane reads 16
// bytes (8 weights) per step, 64 lanes one contiguous KiB; two rows and two steps are in flight
// per wave so that eight 16-byte loads per lane are outstanding.  x is staged once per workgroup
// as bf16 in LDS and read back 16 bytes at a time.
#include <algorithm>
#include "cas_device.hpp"
#include "cas_internal.hpp"

namespace cas {

constexpr int kDenseWaves = 8;

__device__ __forceinline__ float dot8(uint4 w, uint4 x, float acc) {
  const uint32_t wv[4] = {w.x, w.y, w.z, w.w}, xv[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    acc = fmaf(__uint_as_float(wv[e] << 16), __uint_as_float(xv[e] << 16), acc);
    acc = fmaf(__uint_as_float(wv[e] & 0xFFFF0000u), __uint_as_float(xv[e] & 0xFFFF0000u), acc);
  }
  return acc;
}

// cols8 = cols / 8 (cols is a multiple of 8, rows are 16-byte aligned)
__global__ __launch_bounds__(64 * kDenseWaves) void gemv_bf16_kernel(const uint16_t* __restrict__ W, int64_t ld, int rows,
                                                                    int cols8, const uint16_t* __restrict__ x,
                                                                    float* __restrict__ y) {
  extern __shared__ uint4 xs[];  // [cols8]
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < cols8; i += 64 * kDenseWaves) xs[i] = reinterpret_cast<const uint4*>(x)[i];
  __syncthreads();
  const int nw = gridDim.x * kDenseWaves;
  for (int row = blockIdx.x * kDenseWaves + wv; row < rows; row += 2 * nw) {
    const int row1 = row + nw;
    const uint4* w0 = reinterpret_cast<const uint4*>(W + (size_t)row * ld);
    const uint4* w1 = reinterpret_cast<const uint4*>(W + (size_t)(row1 < rows ? row1 : row) * ld);
    float a0 = 0.f, a1 = 0.f;
    int i = lane;
    for (; i + 64 < cols8; i += 128) {
      const uint4 p0 = w0[i], p1 = w0[i + 64], q0 = w1[i], q1 = w1[i + 64];
      const uint4 x0 = xs[i], x1 = xs[i + 64];
      a0 = dot8(p0, x0, a0); a0 = dot8(p1, x1, a0);
      a1 = dot8(q0, x0, a1); a1 = dot8(q1, x1, a1);
    }
    if (i < cols8) {
      const uint4 x0 = xs[i];
      a0 = dot8(w0[i], x0, a0);
      a1 = dot8(w1[i], x0, a1);
    }
    a0 = wave_sum(a0);
    a1 = wave_sum(a1);
    if (lane == 0) {
      y[row] = a0;
      if (row1 < rows) y[row1] = a1;
    }
  }
}

}  // namespace cas

using namespace cas;

extern "C" int cas_gemv_bf16(cas_ctx* ctx, const uint16_t* d_W, int64_t rows, int64_t cols, int64_t ld,
                             const uint16_t* d_x, float* d_y) {
  if (!ctx || rows < 0 || rows > 0x7FFFFFFF || cols < 1 || ld < cols) return CAS_EINVAL;
  if (rows == 0) return CAS_OK;
  if (!d_W || !d_x || !d_y) return CAS_EINVAL;
  // 16-byte loads: whole rows of 8-value pieces
  if ((cols & 7) || (ld & 7) || ((reinterpret_cast<uintptr_t>(d_W) | reinterpret_cast<uintptr_t>(d_x)) & 15)) return CAS_ENOTSUP;
  const size_t lds = (size_t)cols * 2;
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  static LdsLimit lim;
  const int rc = allow_lds(ctx, (const void*)gemv_bf16_kernel, lds, lim);
  if (rc != CAS_OK) return rc;
  // every wave gets at least one pair of rows where there are enough rows; two workgroups per CU
  // at most (1 to 8 measured within 7 % of each other, two best)
  const int64_t want = (rows + 2 * kDenseWaves - 1) / (2 * kDenseWaves);
  const int grid = (int)std::max<int64_t>(1, std::min<int64_t>(want, (int64_t)ctx->num_cu * 2));
  hipLaunchKernelGGL(gemv_bf16_kernel, dim3(grid), dim3(64 * kDenseWaves), lds, ctx->stream, d_W, ld, (int)rows,
                     (int)(cols / 8), d_x, d_y);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}
