/*
 * cassandra.h -- C ABI of the MI355X (gfx950) hot path of Cassandra self-speculative decoding.
 *
 * The operations follow the paper's statement of the method:
 *   - Sec. 4.1: every weight matrix and KV vector is stored as speculation data (the selected
 *     values: sign, exponent, leading mantissa bits, plus a bitmap of their positions) and
 *     verification data (the dropped mantissa bits of the selected values and the unselected
 *     values verbatim).  The draft pass reads speculation data only and pads with zeros; the
 *     target pass reads both and recovers the original bf16 exactly.
 *   - Sec. 4.2: selection = activation-aware magnitude pruning for weights, per-token
 *     magnitude pruning for K and V; truncation = dropping the t low mantissa bits unrounded.
 *   - Sec. 2.2: k draft tokens, one batched verification over k+1 columns, greedy acceptance.
 *   - Sec. 5.1 (encoder): new K/V vectors are formatted online when they are appended.
 *
 * Conventions
 *   - Every function returns CAS_OK (0) or a negative CAS_E* code; no exceptions cross the ABI.
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  All device memory is
 *     allocated and owned by the caller; the library owns only the opaque host structs it
 *     returns and frees them in the matching *_destroy.
 *   - Device work is enqueued on the stream given to cas_ctx_create and is not synchronised;
 *     outputs are valid once the caller synchronises that stream.
 *   - bf16 tensors are passed as uint16_t bit patterns.  Device buffers must be 256-byte aligned.
 *   - One cas_ctx per host thread.
 *   - Empty work (a matrix of 0 rows, 0 tokens to append or read) returns CAS_OK without a
 *     launch; the data pointers of such a call may be NULL.
 */
#ifndef CASSANDRA_H
#define CASSANDRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CAS_OK = 0,
  CAS_EINVAL = -1,   /* bad shape, alignment, format or NULL pointer */
  CAS_ENOTSUP = -2,  /* valid request without a kernel (e.g. exp_mode != 0) */
  CAS_ENOMEM = -3,   /* workspace, pool or the library's fixed scratch array too small */
  CAS_EHIP = -4      /* a HIP call failed; cas_last_hip_error() has the code */
};

typedef struct cas_ctx cas_ctx;

/* Format parameters (Sec. 4.2; defaults of Sec. 7.2.2: 40 % pruned, 4 bits truncated). */
typedef struct {
  int32_t keep_permille; /* kept fraction in 1/1000 (600 = 40 % pruned); K = (keep*G+500)/1000 */
  int32_t trunc_bits;    /* t in 0..7: low mantissa bits moved to the verification data */
  int32_t exp_mode;      /* CAS_EXP_RAW: exponent stored as it is (8 bits).  CAS_EXP_SHARED: one exponent
                            per 32 values (Sec. 4.2, the MX approach), accepted by the KV cache
                            (cas_kv_desc_init); cas_encode_weight takes CAS_EXP_RAW only, the other forms
                            of a matrix are re-codings of its raw encoding (cas_unary_*, cas_mx_*).
                            Anything else: CAS_ENOTSUP. */
} cas_fmt;
enum { CAS_EXP_RAW = 0, CAS_EXP_SHARED = 2 };

/*
 * Layout of one encoded matrix: `rows` selection groups (output rows of a linear layer, or
 * (token, head) vectors of a KV tile) of `cols` values, K kept per row.  Streams are
 * little-endian bit streams in 32-bit words, every row starting on a word boundary:
 *   bitmap : bit c%32 of word c/32 is 1 iff column c is kept        (bw words per row)
 *   spec   : K fields of 16-t bits (word >> t), ascending column     (sw words per row)
 *   lo     : K fields of t bits (word & (2^t-1)), ascending column   (lw words per row)
 *   pruned : cols-K unselected 16-bit words, ascending column        (pw words per row)
 * The speculation buffer holds [bitmap | spec], the verification buffer [lo | pruned], each
 * region 256-byte aligned and followed by 256 bytes of slack that kernels may over-read.
 * The struct is plain data; encoded buffers can be copied or stored verbatim.
 */
typedef struct {
  int64_t rows, cols;
  int32_t K, t;
  int32_t bw, sw, lw, pw;
  int64_t off_bitmap, off_spec;  /* byte offsets inside the speculation buffer */
  int64_t off_lo, off_pruned;    /* byte offsets inside the verification buffer */
  int64_t spec_bytes, verif_bytes; /* sizes the caller must allocate */
} cas_wdesc;

/* ---- context ------------------------------------------------------------------------- */

/* hip_stream: a hipStream_t (NULL = default stream).  d_workspace/ws_bytes: caller-owned
 * device scratch used by calls that say so (attention split partials); may be NULL/0 if
 * those calls are not used. */
int cas_ctx_create(cas_ctx** out, void* hip_stream, void* d_workspace, size_t ws_bytes);
int cas_ctx_destroy(cas_ctx* ctx);
const char* cas_strerror(int code);
int cas_last_hip_error(const cas_ctx* ctx);

/* Measurement hooks.  While enabled, every launch of the four streaming kernels is bracketed
 * by HIP events on the context stream.  kernel_class: 0 draft GEMV, 1 verification GEMM,
 * 2 draft attention, 3 verification attention.  cas_prof_read synchronises the stream and
 * returns the number of launches, the summed kernel time and the summed algorithmic bytes
 * (bytes of the packed streams the launch is obliged to read).  Not for use under graph
 * capture. */
int cas_prof_enable(cas_ctx* ctx, int on);
int cas_prof_read(cas_ctx* ctx, int kernel_class, int64_t* launches, double* total_ms,
                  double* total_bytes);
int cas_prof_reset(cas_ctx* ctx);

/* ---- weights: encode / decode (Sec. 4.2, Sec. 5.1) ------------------------------------ */

/* Host only.  Fills the layout and buffer sizes for a rows x cols matrix. */
int cas_weight_desc(int64_t rows, int64_t cols, const cas_fmt* fmt, cas_wdesc* out);

/* Offline weight formatting.  d_W: bf16 [rows][ld] row-major (ld >= cols, in elements).
 * d_act_norm: float [cols] activation norms a_j >= 0 (score |W_ij| * a_j, one fp32 multiply),
 * or NULL for pure magnitude.  Per row the K highest scores are kept; equal scores go to the
 * lower column.  Writes d_spec (desc->spec_bytes) and d_verif (desc->verif_bytes). */
int cas_encode_weight(cas_ctx* ctx, const uint16_t* d_W, int64_t ld, const float* d_act_norm,
                      const cas_wdesc* desc, void* d_spec, void* d_verif);

/* Reconstruction to dense bf16 [rows][ld] (check/reference path; the step kernels decode in
 * place).  d_verif == NULL: draft reconstruction (kept values with dropped bits 0, others
 * +0, Sec. 4.1).  Otherwise: full reconstruction, bit-identical to the encoded matrix. */
int cas_decode_weight(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec,
                      const void* d_verif, uint16_t* d_out, int64_t ld);

/* ---- stand-alone linear kernels -------------------------------------------------------- */

/* Draft GEMV (Sec. 4.1 draft inference): y[b][r] = sum_c Wdraft[r][c] * x[b][c], fp32
 * accumulation, reading only the speculation buffer.  d_x: bf16 [batch][cols];
 * d_y: float [batch][rows]; batch in 1..4.  x is held in LDS (fp32 for one column, bf16 for a
 * batch): CAS_ENOTSUP if it does not fit (132 bytes per 32 columns for one column, 66 per column
 * of a batch). */
int cas_gemv_draft(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec,
                   const uint16_t* d_x, int batch, float* d_y);

/* The same kernel with the neighbours of a linear layer fused in, as the draft pass of the
 * model uses it (Fig. 2_1 structure).  d_gain != NULL: x is first RMS-normalised,
 * x' = bf16(x * rsqrt(mean(x^2) + eps) * gain), recomputed by every workgroup.  epilogue:
 *   0: d_y[b][r] = W x'                               (d_out16 unused)
 *   1: d_out16[b][r] = bf16(d_out16[b][r] + bf16(W x'))   residual update of a bf16 vector
 *   2: d_out16[b][i] = bf16(silu(bf16(W x')[2i]) * bf16(W x')[2i+1])   SwiGLU over row pairs
 * (rows must be even).  d_y may be NULL for epilogues 1 and 2. */
int cas_gemv_draft_fused(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec,
                         const uint16_t* d_x, int batch, float* d_y, const uint16_t* d_gain,
                         float eps, int epilogue, uint16_t* d_out16);

/* Verification GEMM (Sec. 2.2 batched verification, Sec. 4.1 target inference):
 * Y[c][r] = sum_j W[r][j] * X[c][j] with W the exact bf16 matrix rebuilt from both buffers.
 * d_X: bf16 [ncols][cols]; d_Y: float [ncols][rows]; ncols in 1..32.  The value of a column
 * does not depend on ncols or on the other columns. */
int cas_gemm_verify(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec,
                    const void* d_verif, const uint16_t* d_X, int ncols, float* d_Y);

/* Dense bf16 GEMV on the uncompressed matrix: the BFloat16 baseline the paper's speedups are
 * normalised to (Sec. 7).  d_W: bf16 [rows][ld], d_x: bf16 [cols], d_y: float [rows].  Context
 * for measurements only, not part of the method.  CAS_ENOTSUP unless cols and ld are multiples
 * of 8, d_W and d_x are 16-byte aligned and x fits the LDS. */
int cas_gemv_bf16(cas_ctx* ctx, const uint16_t* d_W, int64_t rows, int64_t cols, int64_t ld,
                  const uint16_t* d_x, float* d_y);

/* ---- speculation data with unary-coded exponents (Sec. 4.2 "Exponent Compression": the
 *      lossless configuration; decoder of Sec. 5.1, zero counting with carry across chunks) ---- */

/*
 * The unary form replaces the spec stream of an encoded matrix; bitmap and verification data
 * stay as they are.  The exponents of the kept values are ranked by frequency over the whole
 * matrix (most frequent first, ties to the smaller exponent, all 256 ranked) and a value of
 * rank r is written as r zero bits followed by a one.  Unary speculation buffer (regions
 * 256-byte aligned, 256 bytes of zeroed slack at the end):
 *   bitmap : as in cas_wdesc                                              (bw words per row)
 *   sm     : K fields of 8-t bits per row: sign, then the 7-t leading mantissa bits,
 *            ascending column, little-endian bit stream                   (smw words per row)
 *   table  : uint8 exp_of_rank[256], then uint8 rank_of_exp[256]
 *   rowoff : uint32 [rows + 1], word index of every row's first code word in ue
 *   ue     : per row its K code words concatenated (first bit of a code at the lower bit
 *            position), rows padded with zeros to a word boundary       (ue_words words)
 * Plain data; buffers can be stored verbatim.
 */
typedef struct {
  cas_wdesc base;   /* the matrix this was re-coded from: rows, cols, K, t, bw, lw, pw, verification offsets */
  int32_t smw;
  int32_t reserved;
  int64_t off_bitmap, off_sm, off_table, off_rowoff, off_ue; /* byte offsets in the unary speculation buffer */
  int64_t ue_words;
  int64_t spec_bytes;           /* size the caller must allocate for the unary speculation buffer */
  uint8_t exp_of_rank[256];     /* the codebook (also stored in the buffer) */
} cas_udesc;

/* Measures an encoded matrix: exponent histogram of its kept values -> codebook -> size of the
 * unary stream.  desc / d_spec: the matrix as written by cas_encode_weight (device).  Needs
 * (rows + 512) * 4 bytes of workspace; synchronises the stream (sizes come back to the host).
 * CAS_ENOMEM if the workspace is too small. */
int cas_unary_plan(cas_ctx* ctx, const cas_wdesc* desc, const void* d_spec, cas_udesc* out);

/* Writes the unary speculation buffer d_uspec (udesc->spec_bytes bytes, 256-byte aligned,
 * device) from the raw one.  udesc must come from cas_unary_plan on the same data.
 * Synchronises the stream once (row offsets are summed on the host). */
int cas_unary_encode(cas_ctx* ctx, const cas_udesc* udesc, const void* d_spec, void* d_uspec);

/* Reconstruction from the unary form (test / reference path): d_verif = NULL gives the draft
 * view (zero padding), otherwise the exact bf16 matrix.  d_out: [rows][ld] words.
 * CAS_ENOTSUP if K bytes of exponents do not fit the LDS of a workgroup. */
int cas_unary_decode(cas_ctx* ctx, const cas_udesc* udesc, const void* d_uspec, const void* d_verif,
                     uint16_t* d_out, int64_t ld);

/* Draft GEMV y = Wdraft x read from the unary speculation buffer alone (Sec. 4.1 draft
 * inference on the Sec. 4.2 lossless format).  d_x: bf16 [cols]; d_y: float [rows].  Same values
 * as cas_gemv_draft on the raw form up to summation order.  CAS_ENOTSUP if x (as fp32) and
 * the exponents of eight rows do not fit the LDS. */
int cas_gemv_draft_unary(cas_ctx* ctx, const cas_udesc* udesc, const void* d_uspec, const uint16_t* d_x,
                         float* d_y);

/* Verification GEMM Y = W X with the speculation data in the unary form (Sec. 4.2 lossless
 * configuration under Sec. 4.1 target inference): W is the exact bf16 matrix, rebuilt from
 * d_uspec + d_verif.  Blocks of rows are first re-coded into the raw spec stream in the
 * workspace, then multiplied by the kernel of cas_gemm_verify, so every output has exactly the
 * bits cas_gemm_verify gives on the raw form.  d_X: bf16 [ncols][cols]; d_Y: float [ncols][rows];
 * 1 <= ncols <= 32.  Workspace: at least 16 rows of the raw stream (16 * sw * 4 + 256 bytes); more
 * means fewer launches.  CAS_ENOMEM if it holds less, CAS_ENOTSUP if K bytes of exponents do
 * not fit the LDS. */
int cas_gemm_verify_unary(cas_ctx* ctx, const cas_udesc* udesc, const void* d_uspec, const void* d_verif,
                          const uint16_t* d_X, int ncols, float* d_Y);

/* ---- speculation data with shared exponents (Sec. 4.2 "Exponent Compression", the MX
 *      approach: the lossy, smaller configuration; decoder of Sec. 5.1, leading-zero count
 *      and shift against the shared exponent) ---- */

/*
 * The shared-exponent form is written from an encoded matrix and keeps its selection.  The
 * paper fixes neither block size, magnitude width nor rounding; this library takes: a block
 * is the 32 columns of one bitmap word; its exponent E is the largest exponent field among
 * the block's kept values (fields 0 and 1 both count as 1; 0 for a block without kept
 * values); a kept value becomes sign + 8-bit magnitude = its significand with the hidden bit
 * written out, shifted right by (E - its exponent), low bits dropped, so that
 * value' = (-1)^sign * magnitude * 2^(E - 134).  Truncation then splits the magnitude: the
 * 8-t leading bits go to the speculation buffer, the t low bits to the verification buffer.
 * Pruned values stay as they are.  Non-finite values are treated as numbers with exponent 255.
 *   MX speculation buffer : bitmap (bw words per row) | sexp (uint8 per bitmap word, ew bytes
 *                           per row, ew = bw rounded up to 4) | field (K fields of 9-t bits:
 *                           sign above the magnitude bits, ascending column; fw words per row)
 *   MX verification buffer: lo (K fields of t bits; lw words per row) | pruned (as cas_wdesc)
 * Regions are 256-byte aligned and followed by 256 bytes of slack.  Plain data.
 */
typedef struct {
  cas_wdesc base;   /* the matrix this was written from: rows, cols, K, t, bw, lw, pw */
  int32_t fw, ew;
  int64_t off_bitmap, off_sexp, off_field;  /* byte offsets in the MX speculation buffer */
  int64_t off_lo, off_pruned;               /* byte offsets in the MX verification buffer */
  int64_t spec_bytes, verif_bytes;          /* sizes the caller must allocate */
} cas_mxdesc;

/* Layout of the shared-exponent form of *desc (host only, no device work). */
int cas_mx_plan(const cas_wdesc* desc, cas_mxdesc* out);

/* Writes both MX buffers (device, 256-byte aligned, sizes from the descriptor) from the raw
 * encoding d_spec / d_verif of the same matrix.  Stream-ordered, no synchronisation. */
int cas_mx_encode(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_spec, const void* d_verif,
                  void* d_mxspec, void* d_mxverif);

/* Reconstruction: d_mxverif = NULL gives the draft view (leading magnitude bits, pruned
 * positions +0), otherwise the converted matrix (all magnitude bits, pruned values merged
 * back).  d_out: [rows][ld] bf16 words. */
int cas_mx_decode(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_mxspec, const void* d_mxverif,
                  uint16_t* d_out, int64_t ld);

/* Draft GEMV y = Wdraft x from the MX speculation buffer alone (Sec. 4.1 draft inference on
 * the shared-exponent format).  d_x: bf16 [cols]; d_y: float [rows].  CAS_ENOTSUP if x does
 * not fit the LDS. */
int cas_gemv_draft_mx(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_mxspec, const uint16_t* d_x,
                      float* d_y);

/* Verification GEMM Y = W' X on the shared-exponent form, W' being the CONVERTED matrix (what
 * cas_mx_decode returns with d_mxverif): the target model of a deployment that uses this
 * format (Sec. 4.2: the conversion is lossy against the original weights, speculation against
 * the converted model stays lossless).  The kernel of cas_gemm_verify with the kept values
 * rebuilt from sign, magnitude and block exponent inside the walk; a column gets the same bits
 * whatever rides along.  d_X: bf16 [ncols][cols]; d_Y: float [ncols][rows]; 1 <= ncols <= 32. */
int cas_gemm_verify_mx(cas_ctx* ctx, const cas_mxdesc* mx, const void* d_mxspec, const void* d_mxverif,
                       const uint16_t* d_X, int ncols, float* d_Y);

/* ---- compressed, paged KV cache (Sec. 4.2 per-token pruning, Sec. 5.1 online encoder) ---- */

/*
 * Geometry of the cache.  The caller fills the first block and calls cas_kv_desc_init, which
 * fills the derived block.  A tile holds the vectors of one (layer, page, K-or-V, kv head):
 * page_tokens rows of head_dim values, K kept per row, streams as in cas_wdesc with row
 * strides bw=4, sw, lw, pw words:
 *   speculation pool tile : [page_tokens][4] bitmap words, then [page_tokens][sw] spec words
 *   verification pool tile: [page_tokens][lw] lo words, then [page_tokens][pw] pruned words
 * Tile index = ((layer * n_pages + page) * 2 + (0 for K, 1 for V)) * n_kv_heads + head; tiles
 * are tile_spec_bytes / tile_verif_bytes apart.  The selection group is one vector of one
 * token and one kv head; K and V are selected separately; ties go to the lower channel.
 *
 * fmt.exp_mode = CAS_EXP_SHARED stores the kept values in the shared-exponent form described at
 * cas_mxdesc, a block being the 32 channels of one bitmap word of one vector: what the cache
 * then holds (and what verification reads back) is the CONVERTED vector, the draft pass reads
 * sign + leading magnitude bits.  Its speculation pool tile is [page_tokens][4] bitmap words,
 * [page_tokens] words with the four block exponents of a vector (block j in byte j), then
 * [page_tokens][sw] words of K fields of 9-t bits; the verification pool tile is unchanged in
 * shape (lo = the t low magnitude bits).
 */
typedef struct {
  int32_t n_layers, n_kv_heads, head_dim /* must be 128 */, page_tokens /* must be 64 */;
  int32_t n_pages, max_seqs, max_pages_per_seq;
  cas_fmt fmt;
  /* derived */
  int32_t K, sw, lw, pw;
  int64_t tile_spec_bytes, tile_verif_bytes;
  int64_t spec_pool_bytes, verif_pool_bytes; /* sizes the caller must allocate */
} cas_kv_desc;

typedef struct cas_kv cas_kv;

/* Host only. */
int cas_kv_desc_init(cas_kv_desc* desc);

/* Binds caller-owned pools and a page table to a cache object.  d_page_table: int32
 * [max_seqs][max_pages_per_seq] of page ids in [0, n_pages), filled by the caller for every
 * position a sequence may reach.  Lengths start at 0 and are kept on the host. */
int cas_kv_create(const cas_kv_desc* desc, void* d_spec_pool, void* d_verif_pool,
                  const int32_t* d_page_table, cas_kv** out);
int cas_kv_destroy(cas_kv* kv);

/* Formats n_tok new vectors and stores them at positions len(seq) .. len(seq)+n_tok-1 of
 * `layer`.  d_K, d_V: bf16 [n_tok][n_kv_heads][head_dim].  Does not change the length: every
 * layer appends at the same positions, then cas_kv_set_len publishes them. */
int cas_kv_append(cas_ctx* ctx, cas_kv* kv, int layer, int seq, const uint16_t* d_K,
                  const uint16_t* d_V, int n_tok);
/* Host only: committed length of a sequence (set: also used to roll back). */
int cas_kv_set_len(cas_kv* kv, int seq, int32_t len);
int cas_kv_len(const cas_kv* kv, int seq, int32_t* len);

/* Reference read-back of positions pos0 .. pos0+n_tok-1 to dense bf16
 * [n_tok][n_kv_heads][head_dim]; full = 0 gives the zero-padded draft view.  The positions must
 * have been written by cas_kv_append (published or not); positions never written read as
 * unspecified values, and a page table entry outside the pool reads as zeros (no access outside
 * the pools either way). */
int cas_kv_read(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int pos0, int n_tok, int full,
                uint16_t* d_K, uint16_t* d_V);

/*
 * Attention of one decode pass for one sequence and layer (Fig. 2_1; Sec. 4.1):
 *   o[c][h] = softmax(q[c][h] . K^T / sqrt(head_dim)) V  over the committed cache positions
 *   and the in-flight vectors 0 .. n_new - ncols + c (causal among the columns).
 * full = 0: cache rebuilt from the speculation pool with zero padding (draft pass);
 * full = 1: cache rebuilt exactly from both pools (verification pass).
 * d_Q: bf16 [ncols][n_q_heads][head_dim] (after the rotary embedding);
 * d_Knew, d_Vnew: bf16 [n_new][n_kv_heads][head_dim], uncompressed, ncols <= n_new <= 64;
 * d_O: bf16 [ncols][n_q_heads][head_dim].  ncols <= 16 and ncols * n_q_heads / n_kv_heads <= 80
 * (48 when full = 0).
 * Uses the context workspace for the per-split partial results (CAS_ENOMEM if too small:
 * splits * n_kv_heads * ncols * group * 132 floats, one split per 64 positions; the model
 * passes run up to four sequences per launch and need the sum of their amounts, each rounded
 * up to 256 bytes).
 * A column's value depends only on the positions it sees: not on ncols, and not on whether an
 * earlier position is already committed or still in flight.
 * The page table is consulted only for pages that hold committed positions (a page of in-flight
 * positions alone needs no entry yet); an entry outside the pool is clamped into it, so a bad
 * table gives wrong values, never an access outside the pools.
 */
int cas_attention(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int full, const uint16_t* d_Q,
                  int ncols, int n_q_heads, const uint16_t* d_Knew, const uint16_t* d_Vnew,
                  int n_new, uint16_t* d_O);

/* cas_attention for n_seqs (1..16) distinct sequences of one layer and one form at once, as the
 * multi-sequence passes issue it (low-batch serving, Sec. 1; Sec. 4.1 for the data each form
 * reads): up to four sequences share one pair of launches.  The h_* arguments are HOST arrays of
 * n_seqs entries; h_d_Q / h_d_Knew / h_d_Vnew / h_d_O hold DEVICE pointers with the shapes of
 * cas_attention for h_ncols[i] columns and h_n_new[i] in-flight vectors.  Every sequence gets bit
 * for bit what cas_attention gives it alone.  Workspace: the partials of the (up to four)
 * sequences of a launch side by side. */
int cas_attention_multi(cas_ctx* ctx, cas_kv* kv, int layer, int n_seqs, const int32_t* h_seqs, int full,
                        const uint16_t* const* h_d_Q, const int32_t* h_ncols, int n_q_heads,
                        const uint16_t* const* h_d_Knew, const uint16_t* const* h_d_Vnew,
                        const int32_t* h_n_new, uint16_t* const* h_d_O);

/*
 * cas_attention for callers that cannot allocate device memory or have none to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit for bit the same output as cas_attention, but the per-split
 * partial results go to a fixed device array inside the library (cas_attention_static_capacity()
 * bytes, 32 MiB, held by every GPU the library runs on until the process ends) instead of the
 * context workspace; the context may have been created without one.  The call allocates
 * nothing (no hipMalloc / hipFree, no events, no library that allocates) and does not
 * synchronise.  CAS_ENOMEM when the partials of the call (splits * n_kv_heads * ncols * group *
 * 132 floats, one split per 64 positions) exceed the array; CAS_EINVAL when the device that was
 * current at cas_ctx_create is not current.  The array keeps the contents of the last call and
 * nothing in it needs clearing (every record is written before it is read); all calls on one GPU
 * share it, so two calls that may overlap on that GPU (different streams or threads) race:
 * serialise them.  The measurement hooks (cas_prof_*) do not see this call.
 */
int cas_attention_static(cas_ctx* ctx, cas_kv* kv, int layer, int seq, int full, const uint16_t* d_Q,
                         int ncols, int n_q_heads, const uint16_t* d_Knew, const uint16_t* d_Vnew,
                         int n_new, uint16_t* d_O);
/* Host only: size in bytes of that array. */
size_t cas_attention_static_capacity(void);

/* ---- model-level steps of one speculative round (Sec. 2.2, Sec. 4.1) --------------------- */

/* Llama-3 style decoder (Fig. 2_1): RMSNorm -> q,k,v projection -> rotary embedding ->
 * grouped-query attention -> output projection -> residual -> RMSNorm -> SwiGLU feed-forward
 * -> residual; final RMSNorm and output head; greedy token = lowest index among the maxima. */
typedef struct {
  int32_t hidden, n_layers, n_q_heads, n_kv_heads, head_dim /* 128 */, ffn, vocab;
  int32_t max_cols; /* columns one pass may carry (1..32); also the number of in-flight K/V slots per
                       sequence and layer.  One sequence contributes at most 16 columns to a pass, and
                       at most 80 / (n_q_heads / n_kv_heads). */
  int32_t max_pos;  /* rows of the rotary table */
  float rms_eps;
  int32_t max_seqs; /* sequences that may have positions in flight at once (0 means 1): every
                       one owns max_cols in-flight K/V slots per layer; sequence ids are < max_seqs */
} cas_model_cfg;

/* One encoded linear layer: layout + the two device buffers (caller-owned). */
typedef struct {
  cas_wdesc desc;
  const void* d_spec;
  const void* d_verif;
} cas_tensor;

/* wqkv: [(n_q_heads + 2 n_kv_heads) * head_dim][hidden], rows ordered q heads, k heads, v heads;
 * wo: [hidden][n_q_heads * head_dim]; wgu: [2 ffn][hidden] with the gate row of unit i at 2i
 * and its up row at 2i+1; wd: [hidden][ffn]; d_g_*: bf16 [hidden] RMSNorm gains. */
typedef struct {
  cas_tensor wqkv, wo, wgu, wd;
  const uint16_t* d_g_attn;
  const uint16_t* d_g_ffn;
} cas_layer_weights;

typedef struct {
  const cas_layer_weights* layers; /* HOST array [n_layers]; copied by cas_model_create */
  cas_tensor lm_head;              /* [vocab][hidden] */
  const uint16_t* d_embed;         /* bf16 [vocab][hidden], not encoded (one row is gathered) */
  const uint16_t* d_g_final;       /* bf16 [hidden] */
  const float* d_rope;             /* float [max_pos][head_dim/2][2] = cos, sin of the position angle */
} cas_model_weights;

typedef struct cas_model cas_model;

/* Host only: bytes of activation scratch cas_model_create needs for this configuration. */
int cas_model_act_bytes(const cas_model_cfg* cfg, size_t* bytes);
/* d_act: caller-owned device block of at least that size (256-byte aligned); it holds the
 * activations of a pass and the uncompressed K/V of the in-flight positions of ONE sequence. */
int cas_model_create(const cas_model_cfg* cfg, const cas_model_weights* weights, void* d_act,
                     size_t act_bytes, cas_model** out);
int cas_model_destroy(cas_model* model);

/* Switches one linear layer of the model to the unary form of its speculation data (Sec. 4.2
 * lossless configuration): from then on draft passes read d_uspec through the kernel of
 * cas_gemv_draft_unary (norm, residual add and SwiGLU run as separate launches with the same
 * roundings) and verification passes through cas_gemm_verify_unary, whose results equal those
 * of the raw form bit for bit; the tensor's raw d_spec is no longer read and may be freed.
 * layer: 0 .. n_layers-1, or -1 for the output head (which is then ignored); which: 0 wqkv,
 * 1 wo, 2 wgu, 3 wd.  udesc / d_uspec: from cas_unary_plan / cas_unary_encode on that tensor
 * (the descriptor is copied, the buffer stays caller-owned); udesc = NULL switches back.
 * CAS_EINVAL if the descriptor does not belong to the tensor.  The context's workspace must
 * hold 16 rows of the largest raw spec stream plus 256 bytes for the verification passes. */
int cas_model_use_unary(cas_model* model, int layer, int which, const cas_udesc* udesc, const void* d_uspec);

/* Switches one linear layer to the shared-exponent form (Sec. 4.2, the MX approach).  The
 * layer's weight is from then on the CONVERTED matrix: draft passes read d_mxspec through the
 * kernel of cas_gemv_draft_mx (with the fused norm / residual / SwiGLU of the raw form),
 * verification passes go through cas_gemm_verify_mx, and a speculative round emits exactly what
 * plain decoding with the converted weights emits.  Arguments as for cas_model_use_unary;
 * mx = NULL switches back; one form at a time per tensor (the last call wins). */
int cas_model_use_mx(cas_model* model, int layer, int which, const cas_mxdesc* mx, const void* d_mxspec,
                     const void* d_mxverif);

/* One draft pass (Sec. 4.1 draft inference): speculation data only for every linear layer and
 * for the cache.  d_token_in: the token at in-flight slot `slot` (position len + slot);
 * its K/V go to slot `slot`, earlier slots must hold the K/V of the previous draft passes of
 * this round.  d_token_out: the drafted next token.  d_logits: NULL or float [vocab].
 * This call and cas_verify_step enqueue kernels only (no copies, no memsets, no
 * synchronisation) and may be recorded into a HIP graph once they have run eagerly with the
 * same shapes; the cache length is an argument of the kernels, so a graph is valid for the
 * cache state it was captured in. */
int cas_draft_step(cas_ctx* ctx, cas_model* model, cas_kv* kv, int seq, const int32_t* d_token_in,
                   int slot, int32_t* d_token_out, float* d_logits);

/* One verification pass (Sec. 2.2, Sec. 4.1 target inference) over k+1 columns: d_tokens =
 * pending token followed by the k drafts, at positions len .. len+k.  Exact weights and cache.
 * d_target[c] = target model's token after column c.  Overwrites in-flight slots 0..k with the
 * target's K/V.  d_logits: NULL or float [k+1][vocab].  k = 0 is plain decoding. */
int cas_verify_step(cas_ctx* ctx, cas_model* model, cas_kv* kv, int seq, const int32_t* d_tokens,
                    int k, int32_t* d_target, float* d_logits);

/* The same passes for several sequences at once (low-batch serving, Sec. 1): the linear
 * layers read their weights once for all columns, attention runs per sequence over its own
 * cache.  h_seqs: n_seqs distinct sequence ids (host).  Draft: one column per sequence, n_seqs
 * in 1..4, h_slots[i] = in-flight slot of sequence i's token, d_tokens_in / d_tokens_out:
 * int32 [n_seqs] (device).  Verification: h_k[i] drafts of sequence i, i.e. h_k[i] + 1 columns;
 * the columns of all sequences, sequence after sequence, are d_tokens / d_target (device).
 * Sequences share a pass while their columns fit max_cols; further sequences go into further
 * passes (each reads the weights again).  Every sequence gets exactly the values the
 * one-sequence calls give it.  Accept and cas_commit stay per sequence. */
int cas_draft_step_multi(cas_ctx* ctx, cas_model* model, cas_kv* kv, int n_seqs, const int32_t* h_seqs,
                         const int32_t* h_slots, const int32_t* d_tokens_in, int32_t* d_tokens_out);
int cas_verify_step_multi(cas_ctx* ctx, cas_model* model, cas_kv* kv, int n_seqs, const int32_t* h_seqs,
                          const int32_t* h_k, const int32_t* d_tokens, int32_t* d_target);

/* After acceptance: format and append the target K/V of the pending token and the n_accepted
 * accepted drafts (slots 0..n_accepted) to every layer of the cache, advance the length by
 * n_accepted + 1, drop the remaining slots. */
int cas_commit(cas_ctx* ctx, cas_model* model, cas_kv* kv, int seq, int n_accepted);

/* One whole round for one sequence: k draft passes chained on the device from `pending`, one
 * verification pass, greedy acceptance, commit.  Synchronises the stream once to read the
 * tokens.  h_out receives n_accepted + 1 tokens; the last one is the next pending token. */
int cas_spec_round(cas_ctx* ctx, cas_model* model, cas_kv* kv, int seq, int32_t pending, int k,
                   int32_t* h_out, int32_t* n_accepted);

/* One speculative round for n_seqs sequences at once (1..4, k + 1 <= max_cols):
 * k multi-sequence draft passes, one multi-sequence verification pass, greedy acceptance and
 * commit per sequence.  h_pending: the pending token of every sequence; h_out: [n_seqs][k+1],
 * row s receives the h_n_accepted[s] + 1 tokens emitted for sequence s. */
int cas_spec_round_multi(cas_ctx* ctx, cas_model* model, cas_kv* kv, int n_seqs, const int32_t* h_seqs,
                         const int32_t* h_pending, int k, int32_t* h_out, int32_t* h_n_accepted);

/* Prefill (functional): runs n prompt tokens through the target path in chunks of as many
 * columns as one sequence may bring to a pass (see max_cols) and commits all of them.  d_tokens: int32 [n] on the device. */
int cas_prefill(cas_ctx* ctx, cas_model* model, cas_kv* kv, int seq, const int32_t* d_tokens, int n);

/* Plain bf16 decode step of the same model from UNCOMPRESSED weights and an uncompressed cache:
 * the BFloat16 baseline the paper's speedups are normalised to (Sec. 6, 7), built from this
 * library's own dense kernels (cas_gemv_bf16, the attention kernels reading plain bf16 rows).
 * Context for measurements, not part of the method; same arithmetic conventions as the encoded
 * passes (bf16 between ops, fp32 inside).  h_layers: HOST array of n_layers entries with DEVICE
 * pointers to the bf16 matrices in the row order of the encoded ones (d_wqkv [q_dim + 2 kv_dim]
 * [hidden], d_wo [hidden][q_dim], d_wgu [2 ffn][hidden] with gate and up rows interleaved, d_wd
 * [hidden][ffn]); gains, embedding and RoPE table are the model's.  d_kcache / d_vcache: bf16
 * [n_layers][max_pos][n_kv_heads][head_dim], positions 0 .. len-1 filled; the step stores the new
 * token's k, v at position len (the caller advances len).  d_logits: NULL or float [vocab].
 * Needs the context's workspace for the attention partials. */
typedef struct cas_dense_layer {
  const uint16_t* d_wqkv;
  const uint16_t* d_wo;
  const uint16_t* d_wgu;
  const uint16_t* d_wd;
} cas_dense_layer;
int cas_dense_decode_step(cas_ctx* ctx, cas_model* model, const cas_dense_layer* h_layers,
                          const uint16_t* d_lm_head, uint16_t* d_kcache, uint16_t* d_vcache, int len,
                          const int32_t* d_token_in, int32_t* d_token_out, float* d_logits);

/* Greedy acceptance (Sec. 2.2).  Host only, no side effects.  h_draft: k drafted tokens;
 * h_target: k+1 target tokens.  n_accepted = number of leading positions where they are
 * identical; h_out receives those n tokens followed by h_target[n] (n+1 tokens). */
int cas_accept(const int32_t* h_draft, const int32_t* h_target, int k, int32_t* n_accepted,
               int32_t* h_out);

/* Rejection-sampling acceptance (Eq. 1).  Host only.  h_p[i], h_q[i]: probability of the
 * (i+1)-th drafted token under the target and the draft model (q > 0); h_r[i]: uniform random
 * numbers in [0, 1) supplied by the caller.  n_accepted = min({i-1 : 1 <= i <= gamma,
 * r_i > p_i / q_i} U {gamma}); the ratio is formed in double precision. */
int cas_accept_sampling(const double* h_p, const double* h_q, const double* h_r, int gamma,
                        int32_t* n_accepted);

/* Probability of a token under the softmax of a row of logits, as Eq. 1 needs it for the drafted
 * tokens (p_i(x) from the target model's logits, q_i(x) from the draft model's).  d_logits: float
 * [n][vocab]; d_tokens: int32 [n]; d_probs: float [n] (0 for a token outside the vocabulary).
 * fp32 with the row maximum subtracted; reductions in a fixed order.  Enqueues one kernel. */
int cas_token_probs(cas_ctx* ctx, const float* d_logits, int vocab, int n, const int32_t* d_tokens,
                    float* d_probs);

/* One whole round with the rejection-sampling acceptance rule (Sec. 2.2, Eq. 1) in place of the
 * greedy one: k draft passes, one verification pass, p_i and q_i of the k drafted tokens from the
 * two sets of logits on the device (cas_token_probs), n from Eq. 1 with the caller's uniform
 * numbers h_r[k] (cas_accept_sampling, ratio in double precision), commit.  Where the paper is
 * silent: the drafted tokens are the draft model's greedy tokens, and the token emitted after
 * the n accepted drafts is the target model's greedy token at that position.  d_scratch: device
 * floats, cas_spec_round_sampling_scratch_floats(vocab, k) of them (the logits of the 2k+1
 * columns and the 2k probabilities), caller-owned.  h_out: n + 1 tokens; h_p, h_q: NULL or
 * double [k], the probabilities used.  Synchronises the stream once. */
size_t cas_spec_round_sampling_scratch_floats(int vocab, int k);
int cas_spec_round_sampling(cas_ctx* ctx, cas_model* model, cas_kv* kv, int seq, int32_t pending, int k,
                            const double* h_r, float* d_scratch, int32_t* h_out, int32_t* n_accepted,
                            double* h_p, double* h_q);

/* Objective of the format search (Eq. 2): acceptance rate per bit the draft model reads,
 *   J = alpha / (S_w (1 - w_p)(B - w_t) + S_kv (1 - kv_p)(B - kv_t)),
 * with the kept fractions 1 - w_p, 1 - kv_p given in 1/1000.  Host only.  s_w, s_kv: numbers of
 * weight and cached values; b_bits: width of the target model's values (16).  Writes J to
 * *h_j.  CAS_EINVAL for a zero denominator or arguments out of range. */
int cas_objective(double alpha, double s_w, int w_keep_permille, int w_trunc_bits, double s_kv,
                  int kv_keep_permille, int kv_trunc_bits, int b_bits, double* h_j);

/* Grid search of Sec. 7.2.2 over the weight format with the cache format fixed: h_alpha is
 * [n_keep][n_trunc], the acceptance rate the caller measured for every pair (keep fraction
 * h_keep_permille[i], truncation h_trunc_bits[j]).  Returns the indices of the pair with the
 * largest J (the first one in row-major order among equals).  Host only. */
int cas_tune_grid(const double* h_alpha, int n_keep, const int32_t* h_keep_permille, int n_trunc,
                  const int32_t* h_trunc_bits, double s_w, double s_kv, int kv_keep_permille,
                  int kv_trunc_bits, int b_bits, int32_t* best_keep_index, int32_t* best_trunc_index);

/* Speed model of Sec. 2.2.  A round of gamma draft passes and one verification pass costs
 * gamma * t_draft + t_verify and emits the accepted drafts plus the target's own next token;
 * with a per-token acceptance probability alpha (reading: the i-th draft is accepted iff drafts
 * 1..i all are, independently with probability alpha each) that is 1 + alpha + ... + alpha^gamma
 * tokens on average.  Plain decoding costs t_plain per token.  Host only; each output may be
 * NULL.  speedup = tokens_per_s * t_plain.  CAS_EINVAL unless 0 <= alpha <= 1, t_verify > 0. */
int cas_speed_model(double alpha, int gamma, double t_draft, double t_verify, double t_plain,
                    double* tokens_per_round, double* tokens_per_s, double* speedup);

/* Format search (Sec. 7.2.2) with MEASURED pass times as the cost of a format in place of Eq. 2's
 * bit count: h_alpha, h_t_draft, h_t_verify are [n_keep][n_trunc] (the acceptance rate the caller
 * measured or assumes for every grid point, and the times of one draft pass and one verification
 * pass of gamma + 1 columns in that format on this machine).  Returns the grid point with the
 * most tokens per second under cas_speed_model (first in row-major order among equals);
 * h_tokens_per_s: NULL or [n_keep][n_trunc], the rate of every point.  Host only. */
int cas_tune_measured(const double* h_alpha, const double* h_t_draft, const double* h_t_verify,
                      int n_keep, int n_trunc, int gamma, int32_t* best_keep_index,
                      int32_t* best_trunc_index, double* h_tokens_per_s);

#ifdef __cplusplus
}
#endif
#endif /* CASSANDRA_H */
