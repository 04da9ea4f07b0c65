// Device-side helpers shared by the gfx950 kernels: wave64 scans through DPP, bit-field
// access to the packed streams, bf16 conversion.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace cas {

constexpr int kWave = 64;

__device__ __forceinline__ int lane_id() { return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// DPP controls (GFX9 encoding)
constexpr int DPP_ROW_SHR1 = 0x111, DPP_ROW_SHR2 = 0x112, DPP_ROW_SHR4 = 0x114, DPP_ROW_SHR8 = 0x118;
constexpr int DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;
constexpr int DPP_QUAD_BCAST0 = 0x00, DPP_QUAD_BCAST3 = 0xFF;

// Inclusive prefix sum over the 64 lanes of a wave.  Lanes whose DPP source is outside the
// row, or that are masked off, add 0.
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, DPP_ROW_SHR1, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, DPP_ROW_SHR2, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, DPP_ROW_SHR4, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, DPP_ROW_SHR8, 0xf, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, DPP_ROW_BCAST15, 0xa, 0xf, false);
  v += __builtin_amdgcn_update_dpp(0, v, DPP_ROW_BCAST31, 0xc, 0xf, false);
  return v;
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_addf(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}

// Sum of v over the wave, returned in every lane (same tree as the scan; lane 63 holds it).
__device__ __forceinline__ float wave_sum(float v) {
  v = dpp_addf<DPP_ROW_SHR1, 0xf>(v);
  v = dpp_addf<DPP_ROW_SHR2, 0xf>(v);
  v = dpp_addf<DPP_ROW_SHR4, 0xf>(v);
  v = dpp_addf<DPP_ROW_SHR8, 0xf>(v);
  v = dpp_addf<DPP_ROW_BCAST15, 0xa>(v);
  v = dpp_addf<DPP_ROW_BCAST31, 0xc>(v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_maxf(float v) {
  // lanes without a source keep their own value (old = v), so the identity is v itself
  return fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK,
                                                              0xf, false)));
}

// Maximum of v over the wave, returned in every lane (same DPP tree as wave_sum).
__device__ __forceinline__ float wave_max(float v) {
  v = dpp_maxf<DPP_ROW_SHR1, 0xf>(v);
  v = dpp_maxf<DPP_ROW_SHR2, 0xf>(v);
  v = dpp_maxf<DPP_ROW_SHR4, 0xf>(v);
  v = dpp_maxf<DPP_ROW_SHR8, 0xf>(v);
  v = dpp_maxf<DPP_ROW_BCAST15, 0xa>(v);
  v = dpp_maxf<DPP_ROW_BCAST31, 0xc>(v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

// float -> bf16, round to nearest even (NaN stays a quiet NaN).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t b = __float_as_uint(f);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x40u);
  return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float round_bf16(float f) { return bf16_to_f32(f32_to_bf16(f)); }

// position of the lowest set bit, -1 if none: exactly what v_ffbl_b32 returns, so no select
__device__ __forceinline__ int lowest_bit(uint32_t m) {
  int r;
  asm("v_ffbl_b32 %0, %1" : "=v"(r) : "v"(m));
  return r;
}

// Read a `width`-bit field (1..32 bits) at bit offset `bit` of a little-endian word stream
// (generic path).  The word after the field's first one is always read as well and the two are
// funnel-shifted: no 64-bit arithmetic, no divergent second load.  Every stream region ends
// with slack, so the extra word is in bounds.
__device__ __forceinline__ uint32_t read_field(const uint32_t* __restrict__ s, uint32_t bit, int width) {
  const uint32_t w = bit >> 5;
  const uint32_t v = __builtin_amdgcn_alignbit(s[w + 1], s[w], bit & 31u);
  return width >= 32 ? v : (v & ((1u << width) - 1u));
}

// Field i (compile-time) of `width` bits from a register window a[] whose bit 0 is field 0.
// Returns the field shifted to the top of a 32-bit word: bits [31 : 32-width].
template <int WIDTH, int I, int NW>
__device__ __forceinline__ uint32_t field_top(const uint32_t (&a)[NW]) {
  constexpr int bit = I * WIDTH, w = bit >> 5, sh = bit & 31;
  if constexpr (sh + WIDTH <= 32) {
    return (a[w] >> sh) << (32 - WIDTH);
  } else {
    return __builtin_amdgcn_alignbit(a[w + 1], a[w], sh) << (32 - WIDTH);
  }
}

// Field i (compile-time) of `width` bits from a register window, right-aligned and masked.
template <int WIDTH, int I, int NW>
__device__ __forceinline__ uint32_t field_at(const uint32_t (&a)[NW]) {
  constexpr int bit = I * WIDTH, w = bit >> 5, sh = bit & 31;
  if constexpr (sh + WIDTH <= 32) {
    return __builtin_amdgcn_ubfe(a[w], sh, WIDTH);
  } else {
    return __builtin_amdgcn_alignbit(a[w + 1], a[w], sh) & ((1u << WIDTH) - 1u);
  }
}

// compile-time loop: f(integral_constant<int, I>) for I in [B, E)
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

// ---- shared-exponent form (Sec. 4.2, the MX approach): value = (-1)^sign * magnitude * 2^(E - 134) ----
// exponent field with 0 read as 1, and the significand with its hidden bit written out
__device__ __forceinline__ int eff_exponent(uint32_t word) { return max((int)((word >> 7) & 0xFFu), 1); }
__device__ __forceinline__ uint32_t significand(uint32_t word) {
  return (word & 0x7Fu) | (((word >> 7) & 0xFFu) ? 0x80u : 0u);
}

// bf16 word of (-1)^sign * mag * 2^(E - 134): shift out the leading zeros of the magnitude and
// take their count off the exponent; subnormal when the exponent runs out
__device__ __forceinline__ uint32_t mx_word(uint32_t sign, int E, uint32_t mag) {
  const int lz = __clz(mag) - 24;  // 8 for mag == 0 (selected away below)
  const int e = E - lz;
  const uint32_t normal = ((uint32_t)e << 7) | ((mag << lz) & 0x7Fu);
  const uint32_t sub = mag << (max(E, 1) - 1);
  const uint32_t v = mag == 0u ? 0u : (e >= 1 ? normal : sub);  // selects, no branches: called per value in walks
  return (sign << 15) | v;
}

// Raw windows of the packed streams at one 32-column bitmap word, before alignment: the words
// that hold the word's kept fields (spec) and their dropped bits (lo) in KeptWindows, those of
// its pruned values in PrunedWindows.  Loading and decoding are separate so the loads of the
// next word can be in flight while the current one is decoded.
//
// decode() hands each (column position, bf16 word) to `write`.  A lane that runs out of bits
// keeps calling write with position -1 and a don't-care value: the caller maps -1 to a dump
// slot.  All 64 lanes of the wave must call it together.
// MX: the kept fields are those of the shared-exponent form (Sec. 4.2, the MX approach): sign
// above the 8-T leading magnitude bits in the spec-side stream, the T low magnitude bits in lo;
// decode() then takes the block's exponent and writes the bf16 word of
// (-1)^sign * magnitude * 2^(E - 134).
template <int T, bool FULL, bool MX = false>
struct KeptWindows {
  static constexpr int FW = MX ? 9 - T : 16 - T;
  static constexpr int LW = T > 0 ? T : 1;
  uint32_t ds[FW + 1];
  uint32_t dl[LW + 1];
  uint32_t shs, shl;

  // p: kept values of the row before this word
  __device__ __forceinline__ void load(uint32_t p, const uint32_t* __restrict__ sp_row,
                                       const uint32_t* __restrict__ lo_row) {
    {
      uint32_t bit = p * FW;
      shs = bit & 31u;
      const uint32_t* src = sp_row + (bit >> 5);
#pragma unroll
      for (int q = 0; q <= FW; ++q) ds[q] = src[q];
    }
    if constexpr (FULL && T > 0) {
      uint32_t bit = p * T;
      shl = bit & 31u;
      const uint32_t* src = lo_row + (bit >> 5);
#pragma unroll
      for (int q = 0; q <= T; ++q) dl[q] = src[q];
    }
  }

  // m: kept mask of the word; shared_exp: the word's shared exponent (MX only)
  template <class W>
  __device__ __forceinline__ void decode(uint32_t m, W&& write, int shared_exp = 0) const {
    uint32_t ws[FW], wl[LW];
#pragma unroll
    for (int q = 0; q < FW; ++q) ws[q] = __builtin_amdgcn_alignbit(ds[q + 1], ds[q], shs);
    if constexpr (FULL && T > 0) {
#pragma unroll
      for (int q = 0; q < T; ++q) wl[q] = __builtin_amdgcn_alignbit(dl[q + 1], dl[q], shl);
    }
    auto kept = [&](auto E) {
      constexpr int e = decltype(E)::value;
      int pos = lowest_bit(m);
      m &= m - 1u;
      uint32_t v = field_at<FW, e>(ws);
      if constexpr (MX) {
        uint32_t mag = (v & ((1u << (8 - T)) - 1u)) << T;
        if constexpr (FULL && T > 0) mag |= field_at<T, e>(wl);
        v = mx_word(v >> (8 - T), shared_exp, mag);
      } else {
        v <<= T;
        if constexpr (FULL && T > 0) v |= field_at<T, e>(wl);
      }
      write(pos, (uint16_t)v);
    };
    auto kept_tail = [&](auto self, auto E) -> void {
      constexpr int e = decltype(E)::value;
      if constexpr (e < 32) {
        if (__builtin_amdgcn_ballot_w64(m != 0u)) {
          kept(std::integral_constant<int, e>{});
          kept(std::integral_constant<int, e + 1>{});
          self(self, std::integral_constant<int, e + 2>{});
        }
      }
    };
    if (__builtin_amdgcn_ballot_w64(m != 0u)) {
      static_for<0, 8>(kept);
      kept_tail(kept_tail, std::integral_constant<int, 8>{});
    }
  }
};

struct PrunedWindows {
  uint32_t dp[17];
  uint32_t shp;

  // u: pruned values of the row before this word
  __device__ __forceinline__ void load(uint32_t u, const uint32_t* __restrict__ pr_row) {
    shp = (u & 1u) << 4;
    const uint32_t* src = pr_row + (u >> 1);
#pragma unroll
    for (int q = 0; q <= 16; ++q) dp[q] = src[q];
  }

  // pm: mask of the word's unselected columns
  template <class W>
  __device__ __forceinline__ void decode(uint32_t pm, W&& write) const {
    uint32_t wp[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) wp[q] = __builtin_amdgcn_alignbit(dp[q + 1], dp[q], shp);
    auto pruned = [&](auto E) {
      constexpr int e = decltype(E)::value;
      int pos = lowest_bit(pm);
      pm &= pm - 1u;
      write(pos, (uint16_t)(wp[e >> 1] >> ((e & 1) * 16)));
    };
    auto pruned_tail = [&](auto self, auto E) -> void {
      constexpr int e = decltype(E)::value;
      if constexpr (e < 32) {
        if (__builtin_amdgcn_ballot_w64(pm != 0u)) {
          pruned(std::integral_constant<int, e>{});
          pruned(std::integral_constant<int, e + 1>{});
          self(self, std::integral_constant<int, e + 2>{});
        }
      }
    };
    pruned_tail(pruned_tail, std::integral_constant<int, 0>{});
  }
};

// Both together (FULL) or the speculation data alone: pm is 0 and unused without FULL.
template <int T, bool FULL, bool MX = false>
struct WordWindows {
  KeptWindows<T, FULL, MX> k;
  PrunedWindows pr;

  __device__ __forceinline__ void load(uint32_t p, uint32_t u, const uint32_t* __restrict__ sp_row,
                                       const uint32_t* __restrict__ lo_row, const uint32_t* __restrict__ pr_row) {
    k.load(p, sp_row, lo_row);
    if constexpr (FULL) pr.load(u, pr_row);
  }

  template <class W>
  __device__ __forceinline__ void decode(uint32_t m, uint32_t pm, W&& write, int shared_exp = 0) const {
    k.decode(m, write, shared_exp);
    if constexpr (FULL) pr.decode(pm, write);
  }
};

// One-shot form: load the windows of a word and decode it.
template <int T, bool FULL, class W>
__device__ __forceinline__ void decode_word(uint32_t m, uint32_t pm, uint32_t p, uint32_t u,
                                            const uint32_t* __restrict__ sp_row, const uint32_t* __restrict__ lo_row,
                                            const uint32_t* __restrict__ pr_row, W&& write) {
  WordWindows<T, FULL> w;
  w.load(p, u, sp_row, lo_row, pr_row);
  w.decode(m, pm, write);
}

template <int CTRL>
__device__ __forceinline__ int quad_dpp(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}

}  // namespace cas
