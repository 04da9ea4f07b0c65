// Speculation data with unary-coded exponents (Sec. 4.2 "Exponent Compression", the lossless
// configuration): re-coding of an encoded matrix, reconstruction, and the draft GEMV that reads
// the unary form directly.
//
// Decoding (Sec. 5.1: zero counting per chunk, then reorganisation across chunk boundaries).
// A wave takes 64 words of a row's code stream at a time, one word per lane.  The popcount of
// a word is the number of codes that end in it, so a prefix sum over the lanes gives the index
// of the first of them.  The rank of a code is the distance from the previous one-bit minus
// one; for the first one-bit of a word the previous one lies in an earlier word: a prefix
// maximum over "position of the last one-bit" of the preceding words supplies it (words without
// a one pass on what they received).  Each lane then walks the ones of its word and writes the
// exponents (codebook lookup) into an LDS array indexed by value number; the bitmap walk that
// follows picks them up together with the sign / mantissa fields.
#include <algorithm>
#include <vector>

#include "cas_device.hpp"
#include "cas_internal.hpp"

namespace cas {

struct UnaryArgs {
  int rows, cols, K, t, bw, sw, smw, lw, pw;
  // raw form (input of the re-coding)
  const uint32_t* bitmap;
  const uint32_t* spec;
  // unary form
  uint32_t* u_bitmap;
  uint32_t* u_sm;
  const uint8_t* table;  // exp_of_rank[256], rank_of_exp[256]
  uint32_t* rowoff;      // [rows + 1]
  uint32_t* ue;
  // verification data
  const uint32_t* lo;
  const uint32_t* pruned;
};

// inclusive prefix maximum over the wave (signed); same DPP tree as the prefix sum
__device__ __forceinline__ int wave_incl_max(int v) {
  constexpr int ID = -0x7fffffff - 1;
  v = max(v, __builtin_amdgcn_update_dpp(ID, v, DPP_ROW_SHR1, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(ID, v, DPP_ROW_SHR2, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(ID, v, DPP_ROW_SHR4, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(ID, v, DPP_ROW_SHR8, 0xf, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(ID, v, DPP_ROW_BCAST15, 0xa, 0xf, false));
  v = max(v, __builtin_amdgcn_update_dpp(ID, v, DPP_ROW_BCAST31, 0xc, 0xf, false));
  return v;
}

// hi field (16-t bits: sign | exponent | 7-t mantissa bits) of kept value e of a raw row
__device__ __forceinline__ uint32_t raw_hi(const uint32_t* sp_row, int e, int t) {
  return read_field(sp_row, (uint32_t)e * (16 - t), 16 - t);
}

// ---- histogram of the exponents of all kept values -------------------------------------------
__global__ __launch_bounds__(256) void unary_hist_kernel(UnaryArgs a, uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
  const int mb = 7 - a.t;
  for (int row = gw; row < a.rows; row += nw) {
    const uint32_t* sp_row = a.spec + (size_t)row * a.sw;
    for (int e = lane; e < a.K; e += 64) atomicAdd(&h[(raw_hi(sp_row, e, a.t) >> mb) & 0xFF], 1u);
  }
  __syncthreads();
  if (h[threadIdx.x]) atomicAdd(&hist[threadIdx.x], h[threadIdx.x]);
}

// ---- words of every row's code stream: ceil(sum(rank + 1) / 32) ------------------------------
__global__ __launch_bounds__(256) void unary_len_kernel(UnaryArgs a, const uint8_t* __restrict__ rank_of_exp,
                                                        uint32_t* __restrict__ len_words) {
  __shared__ uint8_t rk[256];
  rk[threadIdx.x] = rank_of_exp[threadIdx.x];
  __syncthreads();
  const int lane = threadIdx.x & 63, gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
  const int mb = 7 - a.t;
  for (int row = gw; row < a.rows; row += nw) {
    const uint32_t* sp_row = a.spec + (size_t)row * a.sw;
    int bits = 0;
    for (int e = lane; e < a.K; e += 64) bits += rk[(raw_hi(sp_row, e, a.t) >> mb) & 0xFF] + 1;
    const int total = __builtin_amdgcn_readlane(wave_incl_scan(bits), 63);
    if (lane == 0) len_words[row] = (uint32_t)((total + 31) >> 5);
  }
}

// ---- write bitmap copy, sign/mantissa fields and code words of every row ---------------------
// The output regions are zero before this kernel; bits are OR-ed in.
__global__ __launch_bounds__(256) void unary_emit_kernel(UnaryArgs a) {
  __shared__ uint8_t rk[256];
  rk[threadIdx.x] = a.table[256 + threadIdx.x];
  __syncthreads();
  const int lane = threadIdx.x & 63, gw = blockIdx.x * 4 + (threadIdx.x >> 6), nw = gridDim.x * 4;
  const int mb = 7 - a.t, SW = 8 - a.t;
  for (int row = gw; row < a.rows; row += nw) {
    for (int i = lane; i < a.bw; i += 64) a.u_bitmap[(size_t)row * a.bw + i] = a.bitmap[(size_t)row * a.bw + i];
    const uint32_t* sp_row = a.spec + (size_t)row * a.sw;
    uint32_t* sm_row = a.u_sm + (size_t)row * a.smw;
    uint32_t* ue_row = a.ue + a.rowoff[row];
    uint32_t base = 0;  // bits of the codes written so far
    for (int e0 = 0; e0 < a.K; e0 += 64) {
      const int e = e0 + lane;
      const bool valid = e < a.K;
      uint32_t hi = valid ? raw_hi(sp_row, e, a.t) : 0u;
      const int rank = rk[(hi >> mb) & 0xFF];
      const int len = valid ? rank + 1 : 0;
      const int incl = wave_incl_scan(len);
      const uint32_t one = base + (uint32_t)(incl - len) + (uint32_t)rank;  // position of the code's final one
      base += (uint32_t)__builtin_amdgcn_readlane(incl, 63);
      if (valid) {
        atomicOr(&ue_row[one >> 5], 1u << (one & 31u));
        const uint32_t sm = ((hi >> (mb + 8)) << mb) | (hi & ((1u << mb) - 1u));
        const uint32_t bit = (uint32_t)e * SW, sh = bit & 31u;
        atomicOr(&sm_row[bit >> 5], sm << sh);
        if (sh + SW > 32) atomicOr(&sm_row[(bit >> 5) + 1], sm >> (32u - sh));
      }
    }
  }
}

constexpr int kExpSlack = 32;  // bytes behind a row's K exponents: exhausted lanes read them, and a code
                               // stream with more codes than values spills into them instead of beyond

// Exponents of the K kept values of one row into exps[] (LDS, K + kExpSlack bytes), by one
// wave.  ue_row: the row's code words (nw of them); tab: exp_of_rank in LDS.  All 64 lanes must
// call this together.
__device__ __forceinline__ void unary_row_exponents(const uint32_t* __restrict__ ue_row, int nw, int K,
                                                    const uint8_t* tab, uint8_t* exps, int lane) {
  int ebase = 0, prev_end = -1;  // wave-uniform: codes decoded, position of the last one-bit so far
  for (int b0 = 0; b0 < nw; b0 += 64) {
    const int w = b0 + lane;
    uint32_t u = w < nw ? ue_row[w] : 0u;
    const int cnt = __popc(u);
    const int incl = wave_incl_scan(cnt);
    uint8_t* p = exps + min(ebase + incl - cnt, K);  // the lane's codes are consecutive values
    ebase += __builtin_amdgcn_readlane(incl, 63);
    const int last = u ? 32 * w + 31 - __clz(u) : -1;
    const int imax = wave_incl_max(last);
    int pe = __shfl_up(imax, 1, 64);
    if (lane == 0) pe = -1;
    pe = max(pe, prev_end);
    prev_end = max(prev_end, __builtin_amdgcn_readlane(imax, 63));
    int q = pe + 1 - 32 * w;  // first bit after the previous one-bit, relative to this word
    while (__builtin_amdgcn_ballot_w64(u != 0u)) {
      if (u) {
        const int pos = lowest_bit(u);
        u &= u - 1u;
        *p++ = tab[(pos - q) & 255];  // rank = zeros since the previous one-bit
        q = pos + 1;
      }
    }
  }
}

// ---- reconstruction (reference path): one wave per row ---------------------------------------
__global__ __launch_bounds__(64) void unary_decode_kernel(UnaryArgs a, uint16_t* __restrict__ out, int64_t ld,
                                                          int full) {
  extern __shared__ uint8_t lds8[];
  uint8_t* tab = lds8;         // exp_of_rank
  uint8_t* exps = lds8 + 256;  // [K]
  const int lane = threadIdx.x, row = blockIdx.x;
  for (int i = lane; i < 256; i += 64) tab[i] = a.table[i];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const uint32_t o0 = a.rowoff[row], o1 = a.rowoff[row + 1];
  unary_row_exponents(a.ue + o0, (int)(o1 - o0), a.K, tab, exps, lane);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int mb = 7 - a.t, SW = 8 - a.t;
  const uint32_t* bm_row = a.u_bitmap + (size_t)row * a.bw;
  const uint32_t* sm_row = a.u_sm + (size_t)row * a.smw;
  const uint32_t* lo_row = a.lo + (size_t)row * a.lw;
  const uint32_t* pr_row = a.pruned + (size_t)row * a.pw;
  uint16_t* orow = out + (size_t)row * ld;
  int base = 0;  // kept values before this block of words
  for (int w0 = 0; w0 < a.bw; w0 += 64) {
    const int w = w0 + lane;
    uint32_t m = w < a.bw ? bm_row[w] : 0u;
    const int nvalid = a.cols - w * 32;
    const uint32_t valid = nvalid >= 32 ? 0xFFFFFFFFu : (nvalid <= 0 ? 0u : ((1u << nvalid) - 1u));
    uint32_t pm = ~m & valid;
    const int cnt = __popc(m);
    const int incl = wave_incl_scan(cnt);
    int e = base + incl - cnt;
    int u = w * 32 - e;  // pruned values before this word
    base += __builtin_amdgcn_readlane(incl, 63);
    while (m) {
      const int pos = lowest_bit(m);
      m &= m - 1u;
      const uint32_t sm = read_field(sm_row, (uint32_t)e * SW, SW);
      uint32_t word = (((sm >> mb) << (mb + 8)) | ((uint32_t)exps[e] << mb) | (sm & ((1u << mb) - 1u))) << a.t;
      if (full && a.t > 0) word |= read_field(lo_row, (uint32_t)e * a.t, a.t);
      orow[w * 32 + pos] = (uint16_t)word;
      ++e;
    }
    while (pm) {
      const int pos = lowest_bit(pm);
      pm &= pm - 1u;
      orow[w * 32 + pos] = full ? (uint16_t)read_field(pr_row, (uint32_t)u * 16u, 16) : (uint16_t)0;
      ++u;
    }
  }
}

// ---- the raw spec stream of a block of rows, rebuilt from the unary form: one wave per row ------
// After the row's exponents are in LDS every lane assembles whole output words: word w holds the
// bits of the (at most four) fields of 16-t bits that overlap it.
__global__ __launch_bounds__(64) void unary_expand_kernel(UnaryArgs a, int row0, uint32_t* __restrict__ out) {
  extern __shared__ uint8_t lds8[];
  uint8_t* tab = lds8;         // exp_of_rank
  uint8_t* exps = lds8 + 256;  // [K]
  const int lane = threadIdx.x, row = row0 + blockIdx.x;
  for (int i = lane; i < 256; i += 64) tab[i] = a.table[i];
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const uint32_t o0 = a.rowoff[row], o1 = a.rowoff[row + 1];
  unary_row_exponents(a.ue + o0, (int)(o1 - o0), a.K, tab, exps, lane);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  const int mb = 7 - a.t, SW = 8 - a.t, FW = 16 - a.t;
  // the row's sign / mantissa fields come through LDS as well: a field is looked at by up to two
  // output words, and its two words would otherwise be fetched from memory each time
  uint32_t* sm_row = reinterpret_cast<uint32_t*>(lds8 + 256 + (((size_t)a.K + 3) & ~(size_t)3) + kExpSlack);
  {
    const uint32_t* src = a.u_sm + (size_t)row * a.smw;
    for (int i = lane; i < a.smw; i += 64) sm_row[i] = src[i];
    if (lane == 0) sm_row[a.smw] = 0u;  // read_field looks one word ahead
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  uint32_t* orow = out + (size_t)blockIdx.x * a.sw;
  for (int w = lane; w < a.sw; w += 64) {
    uint32_t word = 0;
    for (int e = (32 * w) / FW; e < a.K; ++e) {
      const int bit = e * FW - 32 * w;  // where the field starts, relative to the word (may be negative)
      if (bit >= 32) break;
      const uint32_t sm = read_field(sm_row, (uint32_t)e * SW, SW);
      const uint32_t f = ((sm >> mb) << (mb + 8)) | ((uint32_t)exps[e] << mb) | (sm & ((1u << mb) - 1u));
      word |= bit >= 0 ? f << bit : f >> (-bit);
    }
    orow[w] = word;
  }
}

// ---- draft GEMV from the unary form: eight waves per workgroup, one row per wave --------------
// Per row a wave first decodes the row's exponents into its LDS array, then walks the bitmap
// in chunks of 64 words as the raw-exponent kernel does: a DPP prefix sum gives each lane the
// index of its first kept value, its sign / mantissa fields are one contiguous run that is
// loaded as a register window and aligned once, and step i of the bit walk uses field i of the
// window and exponent i of the lane's run.  x sits in LDS as fp32 in blocks [1 + 32][64 lanes]
// per chunk whose row 0 is 0.0, so a lane that has run out of set bits multiplies by zero, and
// a lane reads only its own 4-byte column of the block (no bank conflicts between lanes).
constexpr int kUnaryWaves = 8;

template <int T>
__global__ __launch_bounds__(64 * kUnaryWaves) void gemv_draft_unary_kernel(UnaryArgs a, const uint16_t* __restrict__ x,
                                                                           float* __restrict__ y, int kpad) {
  constexpr int SW = 8 - T;  // field: sign, then 7 - T mantissa bits
  extern __shared__ uint8_t lds8[];
  const int nseg = ((a.bw + 63) >> 6) << 6;
  uint8_t* tab = lds8;                                           // exp_of_rank
  float* xs = reinterpret_cast<float*>(lds8 + 256);              // [nseg / 64][33][64]
  uint8_t* exps_all = lds8 + 256 + (size_t)nseg * 33 * 4;        // [waves][kpad + kExpSlack]
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid < 256) tab[tid] = a.table[tid];
  for (int sg = tid; sg < nseg; sg += 64 * kUnaryWaves) xs[(sg >> 6) * 33 * 64 + (sg & 63)] = 0.f;
  for (int c = tid; c < nseg * 32; c += 64 * kUnaryWaves)
    xs[((c >> 11) * 33 + 1 + (c & 31)) * 64 + ((c >> 5) & 63)] = c < a.cols ? bf16_to_f32(x[c]) : 0.f;
  uint8_t* exps = exps_all + (size_t)wv * (kpad + kExpSlack);
  // what lies past a row's last exponent must be a finite number's exponent
  for (int i = lane; i < kpad + kExpSlack; i += 64) exps[i] = 0;
  __syncthreads();
  // rows are dealt round-robin to all waves of the grid; a workgroup stages x once
  for (int row = blockIdx.x * kUnaryWaves + wv; row < a.rows; row += gridDim.x * kUnaryWaves) {
    const uint32_t o0 = a.rowoff[row], o1 = a.rowoff[row + 1];
    unary_row_exponents(a.ue + o0, (int)(o1 - o0), a.K, tab, exps, lane);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const uint32_t* bm_row = a.u_bitmap + (size_t)row * a.bw;
    const uint32_t* sm_row = a.u_sm + (size_t)row * a.smw;
    float acc = 0.f;
    int base = 0;
    for (int w0 = 0; w0 < a.bw; w0 += 64) {
      const int w = w0 + lane;
      uint32_t m = w < a.bw ? bm_row[w] : 0u;
      const int cnt = __popc(m);
      const int incl = wave_incl_scan(cnt);
      const int e0 = base + incl - cnt;
      base += __builtin_amdgcn_readlane(incl, 63);
      // window of the lane's fields: SW + 1 words from the word its first field starts in
      const uint32_t bit = (uint32_t)e0 * SW, sh = bit & 31u;
      const uint32_t* src = sm_row + (bit >> 5);
      uint32_t d[SW + 1], win[SW];
#pragma unroll
      for (int j = 0; j <= SW; ++j) d[j] = src[j];
#pragma unroll
      for (int j = 0; j < SW; ++j) win[j] = __builtin_amdgcn_alignbit(d[j + 1], d[j], sh);
      const uint8_t* ex = exps + e0;
      const float* xb = xs + ((w0 >> 6) * 33 + 1) * 64 + lane;
      auto step = [&](auto I) {
        constexpr int i = decltype(I)::value;
        const int pos = lowest_bit(m);
        m &= m - 1u;
        const uint32_t top = field_top<SW, i>(win);  // sign at bit 31, mantissa bits below
        // fp32 pattern of the zero-padded bf16: sign | exponent | leading mantissa bits
        const uint32_t mant = __builtin_amdgcn_ubfe(top, 8, 23);
        const uint32_t bits = (top & 0x80000000u) | ((uint32_t)ex[i] << 23) | mant;
        acc = fmaf(__uint_as_float(bits), xb[pos * 64], acc);
      };
      static_for<0, 16>(step);
      auto tail = [&](auto self, auto I) -> void {
        constexpr int i = decltype(I)::value;
        if constexpr (i < 32) {
          if (__builtin_amdgcn_ballot_w64(m != 0u)) {
            step(std::integral_constant<int, i>{});
            step(std::integral_constant<int, i + 1>{});
            self(self, std::integral_constant<int, i + 2>{});
          }
        }
      };
      tail(tail, std::integral_constant<int, 16>{});
    }
    acc = wave_sum(acc);
    if (lane == 0) y[row] = acc;
    // the next row overwrites exps[]: every lane must be done reading it
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

static UnaryArgs make_uargs(const cas_udesc& u, const void* spec_raw, void* uspec, const void* verif) {
  const cas_wdesc& d = u.base;
  UnaryArgs a{};
  a.rows = (int)d.rows; a.cols = (int)d.cols; a.K = d.K; a.t = d.t;
  a.bw = d.bw; a.sw = d.sw; a.smw = u.smw; a.lw = d.lw; a.pw = d.pw;
  if (spec_raw) {
    a.bitmap = (const uint32_t*)((const char*)spec_raw + d.off_bitmap);
    a.spec = (const uint32_t*)((const char*)spec_raw + d.off_spec);
  }
  if (uspec) {
    char* b = (char*)uspec;
    a.u_bitmap = (uint32_t*)(b + u.off_bitmap);
    a.u_sm = (uint32_t*)(b + u.off_sm);
    a.table = (const uint8_t*)(b + u.off_table);
    a.rowoff = (uint32_t*)(b + u.off_rowoff);
    a.ue = (uint32_t*)(b + u.off_ue);
  }
  if (verif) {
    a.lo = (const uint32_t*)((const char*)verif + d.off_lo);
    a.pruned = (const uint32_t*)((const char*)verif + d.off_pruned);
  }
  return a;
}

int launch_unary_expand(cas_ctx* ctx, const cas_udesc& u, const void* uspec, int64_t row0, int nrows, uint32_t* out) {
  const cas_wdesc& d = u.base;
  if (nrows <= 0 || d.sw == 0) return CAS_OK;
  const size_t lds = 256 + (size_t)((d.K + 3) & ~3) + kExpSlack + ((size_t)u.smw + 1) * 4;  // codebook, exponents, sm fields
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  UnaryArgs a = make_uargs(u, nullptr, const_cast<void*>(uspec), nullptr);
  static LdsLimit lim;
  const int rc = allow_lds(ctx, (const void*)unary_expand_kernel, lds, lim);
  if (rc != CAS_OK) return rc;
  hipLaunchKernelGGL(unary_expand_kernel, dim3((unsigned)nrows), dim3(64), lds, ctx->stream, a, (int)row0, out);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

static int64_t up256(int64_t v) { return (v + 255) / 256 * 256; }
constexpr int64_t kUnarySlack = 256;

static void fill_layout(cas_udesc* u) {
  const cas_wdesc& d = u->base;
  u->smw = (int32_t)(((int64_t)d.K * (8 - d.t) + 31) / 32);
  u->reserved = 0;
  u->off_bitmap = 0;
  u->off_sm = up256(d.rows * d.bw * 4);
  u->off_table = up256(u->off_sm + d.rows * (int64_t)u->smw * 4 + kUnarySlack);
  u->off_rowoff = u->off_table + 512;
  u->off_ue = up256(u->off_rowoff + (d.rows + 1) * 4);
  u->spec_bytes = up256(u->off_ue + u->ue_words * 4 + kUnarySlack);
}

// codebook from the histogram: most frequent first, ties to the smaller exponent
static void build_codebook(const uint32_t* hist, uint8_t* exp_of_rank, uint8_t* rank_of_exp) {
  int order[256];
  for (int i = 0; i < 256; ++i) order[i] = i;
  std::stable_sort(order, order + 256, [&](int x, int y) { return hist[x] > hist[y]; });
  for (int r = 0; r < 256; ++r) {
    exp_of_rank[r] = (uint8_t)order[r];
    rank_of_exp[order[r]] = (uint8_t)r;
  }
}

static int row_grid(cas_ctx* ctx, int64_t rows) {
  return (int)std::max<int64_t>(1, std::min<int64_t>((rows + 3) / 4, (int64_t)ctx->num_cu * 8));
}

// device row lengths (words) -> host, returns their prefix sums in off[rows + 1]
static int row_offsets(cas_ctx* ctx, const UnaryArgs& a, const uint8_t* d_rank, uint32_t* d_len,
                       std::vector<uint32_t>& off) {
  hipLaunchKernelGGL(unary_len_kernel, dim3(row_grid(ctx, a.rows)), dim3(256), 0, ctx->stream, a, d_rank, d_len);
  CAS_HIP(ctx, hipGetLastError());
  std::vector<uint32_t> len(a.rows);
  CAS_HIP(ctx, hipMemcpyAsync(len.data(), d_len, sizeof(uint32_t) * a.rows, hipMemcpyDeviceToHost, ctx->stream));
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));
  off.assign((size_t)a.rows + 1, 0u);
  uint64_t acc = 0;
  for (int r = 0; r < a.rows; ++r) {
    acc += len[r];
    if (acc > 0xFFFFFFFFull) return CAS_EINVAL;  // the code stream is addressed with 32-bit word indices
    off[r + 1] = (uint32_t)acc;
  }
  return CAS_OK;
}

}  // namespace cas

using namespace cas;

extern "C" int cas_unary_plan(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, cas_udesc* out) {
  if (!ctx || !desc || !out || desc->rows < 0 || desc->cols < 1 || desc->t < 0 || desc->t > 7 || desc->K < 0 ||
      desc->K > desc->cols)
    return CAS_EINVAL;
  *out = cas_udesc{};
  out->base = *desc;
  uint32_t hist[256] = {0};
  std::vector<uint32_t> off(1, 0u);
  if (desc->rows > 0 && desc->K > 0) {
    if (!d_spec || !aligned256(d_spec)) return CAS_EINVAL;
    const size_t need = sizeof(uint32_t) * (size_t)(desc->rows + 512);
    if (!ctx->d_ws || ctx->ws_bytes < need) return CAS_ENOMEM;
    uint32_t* d_hist = (uint32_t*)ctx->d_ws;        // [256] counts, then 256 bytes of rank table
    uint8_t* d_rank = (uint8_t*)(d_hist + 256);
    uint32_t* d_len = d_hist + 512;
    UnaryArgs a = make_uargs(*out, d_spec, nullptr, nullptr);
    CAS_HIP(ctx, hipMemsetAsync(d_hist, 0, sizeof(hist), ctx->stream));
    hipLaunchKernelGGL(unary_hist_kernel, dim3(row_grid(ctx, a.rows)), dim3(256), 0, ctx->stream, a, d_hist);
    CAS_HIP(ctx, hipGetLastError());
    CAS_HIP(ctx, hipMemcpyAsync(hist, d_hist, sizeof(hist), hipMemcpyDeviceToHost, ctx->stream));
    CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));
    uint8_t rank_of_exp[256];
    build_codebook(hist, out->exp_of_rank, rank_of_exp);
    CAS_HIP(ctx, hipMemcpyAsync(d_rank, rank_of_exp, 256, hipMemcpyHostToDevice, ctx->stream));
    int rc = row_offsets(ctx, a, d_rank, d_len, off);
    if (rc != CAS_OK) return rc;
  } else {
    uint8_t rank_of_exp[256];
    build_codebook(hist, out->exp_of_rank, rank_of_exp);
    off.assign((size_t)desc->rows + 1, 0u);
  }
  out->ue_words = off.back();
  fill_layout(out);
  return CAS_OK;
}

static int check_udesc(const cas_udesc* u) {
  if (!u) return CAS_EINVAL;
  const cas_wdesc& d = u->base;
  if (d.rows < 0 || d.cols < 1 || d.t < 0 || d.t > 7 || d.K < 0 || d.K > d.cols || u->ue_words < 0) return CAS_EINVAL;
  cas_udesc chk = *u;
  fill_layout(&chk);
  if (chk.smw != u->smw || chk.off_sm != u->off_sm || chk.off_table != u->off_table ||
      chk.off_rowoff != u->off_rowoff || chk.off_ue != u->off_ue || chk.spec_bytes != u->spec_bytes)
    return CAS_EINVAL;
  return CAS_OK;
}

extern "C" int cas_unary_encode(cas_ctx* ctx, const cas_udesc* udesc, const void* d_spec, void* d_uspec) {
  if (!ctx || check_udesc(udesc) != CAS_OK || !d_uspec || !aligned256(d_uspec)) return CAS_EINVAL;
  const cas_wdesc& d = udesc->base;
  CAS_HIP(ctx, hipMemsetAsync(d_uspec, 0, (size_t)udesc->spec_bytes, ctx->stream));
  uint8_t table[512];
  for (int r = 0; r < 256; ++r) {
    table[r] = udesc->exp_of_rank[r];
    table[256 + udesc->exp_of_rank[r]] = (uint8_t)r;
  }
  char* b = (char*)d_uspec;
  CAS_HIP(ctx, hipMemcpyAsync(b + udesc->off_table, table, 512, hipMemcpyHostToDevice, ctx->stream));
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));  // table[] leaves scope
  if (d.rows == 0) return CAS_OK;
  if (!d_spec || !aligned256(d_spec)) return CAS_EINVAL;
  UnaryArgs a = make_uargs(*udesc, d_spec, d_uspec, nullptr);
  std::vector<uint32_t> off((size_t)d.rows + 1, 0u);
  if (d.K > 0) {
    // row lengths go through the rowoff region itself, then come back as prefix sums
    int rc = row_offsets(ctx, a, a.table + 256, a.rowoff, off);
    if (rc != CAS_OK) return rc;
    if ((int64_t)off.back() != udesc->ue_words) return CAS_EINVAL;  // descriptor of other data
  }
  CAS_HIP(ctx, hipMemcpyAsync(a.rowoff, off.data(), sizeof(uint32_t) * off.size(), hipMemcpyHostToDevice, ctx->stream));
  hipLaunchKernelGGL(unary_emit_kernel, dim3(row_grid(ctx, a.rows)), dim3(256), 0, ctx->stream, a);
  CAS_HIP(ctx, hipGetLastError());
  CAS_HIP(ctx, hipStreamSynchronize(ctx->stream));  // off[] leaves scope
  return CAS_OK;
}

extern "C" int cas_unary_decode(cas_ctx* ctx, const cas_udesc* udesc, const void* d_uspec, const void* d_verif,
                                uint16_t* d_out, int64_t ld) {
  if (!ctx || check_udesc(udesc) != CAS_OK || ld < udesc->base.cols) return CAS_EINVAL;
  const cas_wdesc& d = udesc->base;
  if (d.rows == 0) return CAS_OK;
  if (!d_uspec || !d_out || !aligned256(d_uspec) || !aligned256(d_verif)) return CAS_EINVAL;
  const size_t lds = 256 + (size_t)((d.K + 3) & ~3) + kExpSlack;
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  UnaryArgs a = make_uargs(*udesc, nullptr, const_cast<void*>(d_uspec), d_verif);
  static LdsLimit lim;
  const int rc = allow_lds(ctx, (const void*)unary_decode_kernel, lds, lim);
  if (rc != CAS_OK) return rc;
  hipLaunchKernelGGL(unary_decode_kernel, dim3((unsigned)d.rows), dim3(64), lds, ctx->stream, a, d_out, ld,
                     d_verif ? 1 : 0);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

extern "C" int cas_gemm_verify_unary(cas_ctx* ctx, const cas_udesc* udesc, const void* d_uspec, const void* d_verif,
                                     const uint16_t* d_X, int ncols, float* d_Y) {
  if (!ctx || check_udesc(udesc) != CAS_OK || ncols < 1 || ncols > 32) return CAS_EINVAL;
  if (udesc->base.rows == 0) return CAS_OK;
  if (!d_uspec || !d_verif || !d_X || !d_Y || !aligned256(d_uspec) || !aligned256(d_verif)) return CAS_EINVAL;
  return launch_gemm_verify_unary_fused(ctx, *udesc, d_uspec, d_verif, d_X, ncols, d_Y, 0, nullptr);
}

template <int T>
static int launch_unary_gemv(cas_ctx* ctx, const UnaryArgs& a, const uint16_t* d_x, float* d_y, int kpad, int grid,
                             size_t lds) {
  static LdsLimit lim;
  const int rc = allow_lds(ctx, (const void*)gemv_draft_unary_kernel<T>, lds, lim);
  if (rc != CAS_OK) return rc;
  hipLaunchKernelGGL(gemv_draft_unary_kernel<T>, dim3(grid), dim3(64 * kUnaryWaves), lds, ctx->stream, a, d_x, d_y, kpad);
  CAS_HIP(ctx, hipGetLastError());
  return CAS_OK;
}

extern "C" int cas_gemv_draft_unary(cas_ctx* ctx, const cas_udesc* udesc, const void* d_uspec, const uint16_t* d_x,
                                    float* d_y) {
  if (!ctx || check_udesc(udesc) != CAS_OK) return CAS_EINVAL;
  const cas_wdesc& d = udesc->base;
  if (d.rows == 0) return CAS_OK;
  if (!d_uspec || !d_x || !d_y || !aligned256(d_uspec)) return CAS_EINVAL;
  const int kpad = (d.K + 15) & ~15;
  const size_t nseg = (size_t)((d.bw + 63) / 64 * 64);
  const size_t lds = 256 + nseg * 33 * sizeof(float) + (size_t)kUnaryWaves * (kpad + kExpSlack);
  if (lds > (size_t)ctx->lds_max) return CAS_ENOTSUP;
  UnaryArgs a = make_uargs(*udesc, nullptr, const_cast<void*>(d_uspec), nullptr);
  // as many workgroups as stay resident: every one of them stages x once
  const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(4, (size_t)ctx->lds_max / lds));
  const int grid = (int)std::min<int64_t>((d.rows + kUnaryWaves - 1) / kUnaryWaves, (int64_t)ctx->num_cu * per_cu);
#define CAS_T(TV) case TV: return launch_unary_gemv<TV>(ctx, a, d_x, d_y, kpad, grid, lds);
  switch (d.t) {
    CAS_T(0) CAS_T(1) CAS_T(2) CAS_T(3) CAS_T(4) CAS_T(5) CAS_T(6) CAS_T(7)
  }
#undef CAS_T
  return CAS_EINVAL;
}
