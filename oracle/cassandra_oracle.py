"""Plain CPU oracle for the Cassandra self-speculative decode path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
what the path computes, written from the paper; the HIP library shares no code
with it and never calls it.  Only tests/, the smoke check and the bench's
cpu_baseline leg may import it.

Every function cites the passage of the paper it follows (section / equation /
figure).  Floating point is float64 unless stated; bf16 tensors are uint16 bit
patterns.  Nothing here is blocked, fused or reordered beyond the definition.

Parity pins (tests/test_oracle_*.py): exhaustive bit-exact round trip over all
65536 bf16 patterns, bit-prefix property of truncation, kept count, brute-force
subset search for the selection, closed-form stream sizes, library matmul /
attention special cases, brute-force acceptance, speculative == plain token
streams, hand-worked roundings of the residual add, tied maxima of the greedy token, Eq. 2 and
the grid search worked by hand, the forward composition (target and draft pass) against a
separately written float64 decoder made of library operations, and for the unary exponent code the printed code words, a sequential
scan, the closed-form length and an exhaustive search over code assignments; for the
shared-exponent form the conversion restated as real arithmetic, the lossless special case,
the error bound of one unit of the block's last place and hand-worked blocks.  Parity unpinned:
block size, magnitude width and rounding of the shared-exponent form (the paper fixes none of
them; the reading taken is stated at the functions); acceptance *rates* and speedups (the paper's tables
for them are images that did not survive, and need trained weights).
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

BF16_BITS = 16  # 1 sign + 8 exponent + 7 mantissa (Sec. 4.2, "Exponent Compression")


# ----------------------------------------------------------------------------
# bf16 <-> float helpers
# ----------------------------------------------------------------------------
def bf16_to_f64(u16):
    """Exact widening of bf16 bit patterns to float64."""
    u = np.asarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_to_bf16(x):
    """Round a real value to bf16, nearest-even (via float32; both roundings RNE)."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    b = np.ascontiguousarray(f).view(np.uint32).astype(np.uint64)
    nan = np.isnan(f)
    r = ((b + np.uint64(0x7FFF) + ((b >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16))
    r = np.where(nan, (b >> np.uint64(16)) | np.uint64(0x40), r)
    return r.astype(np.uint16)


def round_bf16(x):
    """Value of x after rounding to bf16 (as float64)."""
    return bf16_to_f64(f64_to_bf16(x))


# ----------------------------------------------------------------------------
# Selection (Sec. 4.2 "Unstructured Value Pruning")
# ----------------------------------------------------------------------------
def kept_count(group: int, keep_permille: int) -> int:
    """Number of kept values in a group of `group` elements."""
    k = (keep_permille * group + 500) // 1000
    return max(0, min(group, k))


def weight_scores(w_u16, act_norm=None):
    """Importance score bits of every weight.

    With activation norms a_j: score = |W_ij| * a_j as one float32 multiply
    (activation-aware rule of Sec. 4.2), compared by its uint32 pattern.
    Without: the 15-bit magnitude pattern of the bf16 (pure magnitude).
    """
    w = np.asarray(w_u16, dtype=np.uint16)
    mag = (w & np.uint16(0x7FFF))
    if act_norm is None:
        return mag.astype(np.uint32)
    a = np.asarray(act_norm, dtype=np.float32)
    absw = (mag.astype(np.uint32) << np.uint32(16)).view(np.float32)
    with np.errstate(invalid="ignore", over="ignore"):
        s = (absw * a[None, :]).astype(np.float32)
    bits = s.view(np.uint32).copy()
    bits[np.isnan(s)] = np.uint32(0x7FFFFFFF)
    return bits


def kv_scores(v_u16):
    """Per-token magnitude score for KV vectors (Sec. 4.2): the 15-bit magnitude."""
    return (np.asarray(v_u16, dtype=np.uint16) & np.uint16(0x7FFF)).astype(np.uint32)


def select_topk(score_bits, k: int):
    """Keep the k highest scores of each row (last axis); equal scores go to the
    lower index.  Returns a bool mask of the same shape."""
    s = np.asarray(score_bits, dtype=np.uint32)
    g = s.shape[-1]
    flat = s.reshape(-1, g)
    mask = np.zeros(flat.shape, dtype=bool)
    if k <= 0:
        return mask.reshape(s.shape)
    # total order: higher score first, then lower index first
    key = (flat.astype(np.uint64) << np.uint64(32)) | (np.uint64(g - 1) - np.arange(g, dtype=np.uint64))[None, :]
    order = np.argsort(key, axis=1, kind="stable")  # ascending; keys are unique
    top = order[:, g - k:]
    np.put_along_axis(mask, top, True, axis=1)
    return mask.reshape(s.shape)


# ----------------------------------------------------------------------------
# Truncation / split (Sec. 4.2 "Mantissa Truncation", Sec. 4.1)
# ----------------------------------------------------------------------------
def split_word(w_u16, t: int):
    """hi = the 16-t leading bits (sign, exponent, leading mantissa bits), lo = the t
    dropped mantissa bits.  No rounding: hi is a bit-prefix of the word."""
    w = np.asarray(w_u16, dtype=np.uint16)
    hi = (w >> np.uint16(t)).astype(np.uint16)
    lo = (w & np.uint16((1 << t) - 1)).astype(np.uint16)
    return hi, lo


# ----------------------------------------------------------------------------
# Packed representation: bitmap + speculation stream + verification streams
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Packed:
    """One matrix whose rows are selection groups with exactly K kept values each.

    bitmap[r, c//32] bit c%32       : column c of row r is kept (Sec. 5.1, bitmap
                                      de-sparsification)
    spec[r]   : K fields of 16-t bits, ascending column order, field e at bit e*(16-t)
    lo[r]     : K fields of t bits (the truncated mantissa bits of the kept values)
    pruned[r] : cols-K full 16-bit words (the unselected values, ascending column)
    Streams are little-endian bit streams stored in uint32 words; each row starts
    on a word boundary.  spec (+bitmap) is the speculation data, lo+pruned the
    verification data (Sec. 4.1).
    """
    rows: int
    cols: int
    K: int
    t: int
    bitmap: np.ndarray
    spec: np.ndarray
    lo: np.ndarray
    pruned: np.ndarray


def _words(bits: int) -> int:
    return (bits + 31) // 32


def stream_words(cols: int, K: int, t: int):
    """(bitmap, spec, lo, pruned) words per row; closed form of the byte accounting
    behind Eq. 2's denominator, plus the bitmap the equation leaves out."""
    return _words(cols), _words(K * (BF16_BITS - t)), _words(K * t), _words((cols - K) * 16)


def _pack_fields(fields, width: int, nwords: int):
    """fields [rows, m] of `width` bits -> uint32 [rows, nwords] little-endian bit stream."""
    rows, m = fields.shape
    if nwords == 0:
        return np.zeros((rows, 0), dtype=np.uint32)
    out = np.zeros((rows, nwords * 32), dtype=np.uint8)
    if m and width:
        f = fields.astype(np.uint32)
        bits = ((f[:, :, None] >> np.arange(width, dtype=np.uint32)[None, None, :]) & 1).astype(np.uint8)
        out[:, : m * width] = bits.reshape(rows, m * width)
    packed = np.packbits(out, axis=1, bitorder="little")
    return np.ascontiguousarray(packed).view("<u4").astype(np.uint32)


def _unpack_fields(words, width: int, m: int):
    rows = words.shape[0]
    if m == 0 or width == 0:
        return np.zeros((rows, m), dtype=np.uint16)
    by = np.ascontiguousarray(words.astype("<u4")).view(np.uint8)
    bits = np.unpackbits(by, axis=1, bitorder="little")[:, : m * width].reshape(rows, m, width)
    weights = (1 << np.arange(width, dtype=np.uint32))
    return (bits.astype(np.uint32) * weights[None, None, :]).sum(axis=2).astype(np.uint16)


def pack(w_u16, mask, t: int) -> Packed:
    """Write the split of Sec. 4.1/4.2 into the packed streams."""
    w = np.asarray(w_u16, dtype=np.uint16)
    rows, cols = w.shape
    counts = mask.sum(axis=1)
    K = int(counts[0]) if rows else 0
    assert (counts == K).all(), "every row must keep the same number of values"
    bw, sw, lw, pw = stream_words(cols, K, t)
    hi, lo = split_word(w, t)
    # row-major boolean indexing keeps ascending column order inside each row
    hi_k = hi[mask].reshape(rows, K)
    lo_k = lo[mask].reshape(rows, K)
    pr = w[~mask].reshape(rows, cols - K)
    bm = np.zeros((rows, bw * 32), dtype=np.uint8)
    bm[:, :cols] = mask
    bitmap = np.ascontiguousarray(np.packbits(bm, axis=1, bitorder="little")).view("<u4").astype(np.uint32)
    return Packed(rows, cols, K, t, bitmap,
                  _pack_fields(hi_k, BF16_BITS - t, sw),
                  _pack_fields(lo_k, t, lw),
                  _pack_fields(pr, 16, pw))


def unpack_mask(p: Packed):
    by = np.ascontiguousarray(p.bitmap.astype("<u4")).view(np.uint8)
    return np.unpackbits(by, axis=1, bitorder="little")[:, : p.cols].astype(bool)


def decode_draft(p: Packed):
    """Draft reconstruction (Sec. 4.1): speculation data with zero padding -- kept
    values get their leading bits back with the dropped mantissa bits as 0, pruned
    positions read +0."""
    mask = unpack_mask(p)
    hi = _unpack_fields(p.spec, BF16_BITS - p.t, p.K)
    out = np.zeros((p.rows, p.cols), dtype=np.uint16)
    out[mask] = (hi.astype(np.uint32) << p.t).astype(np.uint16).reshape(-1)
    return out


def decode_full(p: Packed):
    """Target reconstruction (Sec. 4.1, Sec. 5.1 mantissa concatenation): leading and
    dropped mantissa bits concatenated, pruned values merged back through the bitmap."""
    mask = unpack_mask(p)
    hi = _unpack_fields(p.spec, BF16_BITS - p.t, p.K)
    lo = _unpack_fields(p.lo, p.t, p.K)
    pr = _unpack_fields(p.pruned, 16, p.cols - p.K)
    out = np.zeros((p.rows, p.cols), dtype=np.uint16)
    out[mask] = ((hi.astype(np.uint32) << p.t) | lo).astype(np.uint16).reshape(-1)
    out[~mask] = pr.reshape(-1)
    return out


def encode_weight(w_u16, keep_permille: int, t: int, act_norm=None) -> Packed:
    """Offline weight formatting (Sec. 5.1 last paragraph): per output row, keep the
    K best-scoring inputs (Sec. 4.2), truncate, split, pack."""
    w = np.asarray(w_u16, dtype=np.uint16)
    K = kept_count(w.shape[1], keep_permille)
    mask = select_topk(weight_scores(w, act_norm), K)
    return pack(w, mask, t)


def encode_kv(v_u16, keep_permille: int, t: int) -> Packed:
    """Online KV formatting (Sec. 5.1 encoder, Sec. 4.2 per-token magnitude pruning):
    rows are (token, head) vectors of head_dim values; K largest magnitudes kept."""
    v = np.asarray(v_u16, dtype=np.uint16)
    K = kept_count(v.shape[1], keep_permille)
    mask = select_topk(kv_scores(v), K)
    return pack(v, mask, t)


# ----------------------------------------------------------------------------
# Unary-coded exponents: the lossless "Cassandra-1" speculation data (Sec. 4.2
# "Exponent Compression", decoder of Sec. 5.1 / Algorithm 1)
# ----------------------------------------------------------------------------
def unary_codebook(exps):
    """Codebook of the unary code: exponents ranked by how often they occur among the kept
    values of the tensor, the most frequent first (Sec. 4.2: more frequent exponents get
    fewer bits).  All 256 exponents are ranked, ties by the smaller exponent, so every value
    stays encodable.  Returns (exp_of_rank, rank_of_exp), uint8[256] each."""
    counts = np.bincount(np.asarray(exps, dtype=np.int64).reshape(-1), minlength=256)
    order = sorted(range(256), key=lambda e: (-int(counts[e]), e))
    exp_of_rank = np.array(order, dtype=np.uint8)
    rank_of_exp = np.zeros(256, dtype=np.uint8)
    rank_of_exp[exp_of_rank] = np.arange(256, dtype=np.uint8)
    return exp_of_rank, rank_of_exp


def unary_encode_bits(ranks):
    """Rank r -> r zeros followed by a one (Sec. 4.2: 1, 01, 001, ...), codes concatenated in
    order.  Returns the bit sequence (uint8 0/1), first bit first."""
    out = []
    for r in np.asarray(ranks, dtype=np.int64).reshape(-1):
        out.extend([0] * int(r))
        out.append(1)
    return np.array(out, dtype=np.uint8)


def unary_decode_chunked(bits, numel: int):
    """Decoder of Sec. 5.1: the stream is cut into 8-bit chunks; every chunk counts, for each
    of its ones, the zeros since the previous one inside the chunk (parallel zero counter) and
    remembers the zeros after its last one; the reorganisation step then adds to the first
    count of a chunk the zeros that the preceding chunks left open (a chunk without a one
    passes on what it received plus its 8 zeros).  Stops after numel codes."""
    b = np.asarray(bits, dtype=np.uint8).reshape(-1)
    pad = (-len(b)) % 8
    chunks = np.concatenate([b, np.zeros(pad, dtype=np.uint8)]).reshape(-1, 8)
    outputs, trailing = [], []
    for ch in chunks:                      # zero counting, independent per chunk
        cnt, outs = 0, []
        for bit in ch:
            if bit == 0:
                cnt += 1
            else:
                outs.append(cnt)
                cnt = 0
        outputs.append(outs)
        trailing.append(cnt)
    carry = 0                              # reorganisation across chunk boundaries
    for k, outs in enumerate(outputs):
        if outs:
            outs[0] += carry
            carry = trailing[k]
        else:
            carry += trailing[k]
    ranks = [r for outs in outputs for r in outs]
    assert len(ranks) >= numel, "stream holds fewer codes than values"
    return np.array(ranks[:numel], dtype=np.int64)


@dataclasses.dataclass
class PackedUnary:
    """Speculation data with unary-coded exponents.  base holds the bitmap and the
    verification streams (lo, pruned) unchanged; its spec stream is replaced by
      sm[r]  : K fields of 8-t bits = sign, then the 7-t leading mantissa bits
      ue     : for each row the K unary codes of its kept values' exponent ranks, ascending
               column order, as a little-endian bit stream; row r occupies the words
               ue_off[r] .. ue_off[r+1]-1 (rows start on word boundaries, zero padded)
      exp_of_rank : the codebook."""
    base: Packed
    sm: np.ndarray
    ue: np.ndarray
    ue_off: np.ndarray
    exp_of_rank: np.ndarray


def _split_hi(hi, t: int):
    """hi field (16-t bits: sign | exponent | 7-t mantissa bits) -> (sm, exponent)."""
    mb = 7 - t
    h = hi.astype(np.uint32)
    exp = (h >> mb) & 0xFF
    sm = ((h >> (mb + 8)) << mb) | (h & ((1 << mb) - 1))
    return sm.astype(np.uint16), exp.astype(np.uint16)


def to_unary(p: Packed) -> PackedUnary:
    """Re-code the speculation stream of a packed matrix with unary exponents (Sec. 4.2; the
    paper applies the exponent coding to the speculation group only, Sec. 5.1 encoder)."""
    hi = _unpack_fields(p.spec, BF16_BITS - p.t, p.K)
    sm, exp = _split_hi(hi, p.t)
    exp_of_rank, rank_of_exp = unary_codebook(exp)
    ranks = rank_of_exp[exp]
    rows_words, off = [], [0]
    for r in range(p.rows):
        bits = unary_encode_bits(ranks[r])
        nw = _words(len(bits))
        padded = np.zeros(nw * 32, dtype=np.uint8)
        padded[: len(bits)] = bits
        rows_words.append(np.ascontiguousarray(np.packbits(padded, bitorder="little")).view("<u4").astype(np.uint32))
        off.append(off[-1] + nw)
    ue = np.concatenate(rows_words) if rows_words else np.zeros(0, dtype=np.uint32)
    return PackedUnary(p, _pack_fields(sm, 8 - p.t, _words(p.K * (8 - p.t))), ue,
                       np.array(off, dtype=np.uint32), exp_of_rank)


def _hi_from_unary(u: PackedUnary):
    p = u.base
    mb = 7 - p.t
    sm = _unpack_fields(u.sm, 8 - p.t, p.K).astype(np.uint32)
    hi = np.zeros((p.rows, p.K), dtype=np.uint32)
    for r in range(p.rows):
        words = u.ue[int(u.ue_off[r]): int(u.ue_off[r + 1])]
        bits = np.unpackbits(np.ascontiguousarray(words.astype("<u4")).view(np.uint8), bitorder="little")
        exp = u.exp_of_rank[unary_decode_chunked(bits, p.K)].astype(np.uint32) if p.K else np.zeros(0, np.uint32)
        hi[r] = ((sm[r] >> mb) << (mb + 8)) | (exp << mb) | (sm[r] & ((1 << mb) - 1))
    return hi


def decode_draft_unary(u: PackedUnary):
    """Draft reconstruction from the unary-coded speculation data: identical in value to
    decode_draft of the raw-exponent form (the exponent coding is lossless, Sec. 4.2)."""
    p = u.base
    out = np.zeros((p.rows, p.cols), dtype=np.uint16)
    out[unpack_mask(p)] = (_hi_from_unary(u) << p.t).astype(np.uint16).reshape(-1)
    return out


def decode_full_unary(u: PackedUnary):
    p = u.base
    mask = unpack_mask(p)
    lo = _unpack_fields(p.lo, p.t, p.K)
    pr = _unpack_fields(p.pruned, 16, p.cols - p.K)
    out = np.zeros((p.rows, p.cols), dtype=np.uint16)
    out[mask] = ((_hi_from_unary(u) << p.t) | lo).astype(np.uint16).reshape(-1)
    out[~mask] = pr.reshape(-1)
    return out


def gemv_draft_unary(u: PackedUnary, x_u16):
    return gemv(decode_draft_unary(u), x_u16)


# ----------------------------------------------------------------------------
# Shared-exponent (MX) form of the speculation group (Sec. 4.2 "Exponent Compression",
# first approach; decoder #N of Sec. 5.1; the lossy configuration, Cassandra-2)
# ----------------------------------------------------------------------------
MX_BLOCK = 32   # consecutive columns of a row that share one exponent
MX_MAG_BITS = 8  # the bf16 significand with its hidden bit written out


def _bf16_parts(w_u16):
    """(sign, effective exponent, 8-bit significand): value = (-1)^s * sig * 2^(e - 134).
    Subnormals and zeros have no hidden bit and exponent 1."""
    w = np.asarray(w_u16, dtype=np.uint16).astype(np.int64)
    exp = (w >> 7) & 0xFF
    frac = w & 0x7F
    return w >> 15, np.maximum(exp, 1), np.where(exp > 0, 0x80 | frac, frac)


def mx_shared_exponents(w_u16, mask):
    """Shared exponent of every block of MX_BLOCK columns: the largest exponent among its
    kept values (0 for a block without kept values).  [rows, ceil(cols/32)] uint8."""
    w = np.asarray(w_u16, dtype=np.uint16)
    rows, cols = w.shape
    nb = (cols + MX_BLOCK - 1) // MX_BLOCK
    _, e, _ = _bf16_parts(w)
    ek = np.zeros((rows, nb * MX_BLOCK), dtype=np.int64)
    ek[:, :cols] = np.where(mask, e, 0)
    return ek.reshape(rows, nb, MX_BLOCK).max(axis=2).astype(np.uint8)


def mx_magnitudes(w_u16, mask, sexp):
    """Sign and 8-bit magnitude of every kept value against its block's exponent: the
    significand shifted right by the exponent difference, low bits dropped (no rounding,
    as for the mantissa truncation of Sec. 4.2).  Entries outside the mask are 0."""
    w = np.asarray(w_u16, dtype=np.uint16)
    cols = w.shape[1]
    s, e, sig = _bf16_parts(w)
    E = np.repeat(sexp.astype(np.int64), MX_BLOCK, axis=1)[:, :cols]
    shift = np.clip(E - e, 0, MX_MAG_BITS)
    mag = np.where(mask, sig >> shift, 0)
    return np.where(mask, s, 0).astype(np.uint16), mag.astype(np.uint16)


def mx_to_bf16(sign, E, mag):
    """Decoder #N of Sec. 5.1 for one value: count the leading zeros of the magnitude, shift
    them out, subtract the count from the shared exponent.  The result is exactly
    (-1)^s * mag * 2^(E - 134), always a bf16 value (subnormal when the exponent runs out)."""
    sign, E, mag = int(sign), int(E), int(mag)
    if mag == 0:
        return sign << 15
    lz = MX_MAG_BITS - mag.bit_length()
    e = E - lz
    if e >= 1:
        return (sign << 15) | (e << 7) | ((mag << lz) & 0x7F)
    return (sign << 15) | (mag << (E - 1))


@dataclasses.dataclass
class PackedMX:
    """Shared-exponent form of a packed matrix.  base supplies bitmap and pruned stream;
      sexp[r, b] : shared exponent of block b (the 32 columns of bitmap word b)
      field[r]   : K fields of 9-t bits = sign, then the 8-t leading magnitude bits
      lo[r]      : K fields of t bits, the dropped magnitude bits (verification data)."""
    base: Packed
    sexp: np.ndarray
    field: np.ndarray
    lo: np.ndarray


def to_mx(p: Packed) -> PackedMX:
    """Exponent sharing first, truncation second (the order Sec. 4.2 states): the kept
    values of a packed matrix -> shared exponents, sign+magnitude split at t bits."""
    mask = unpack_mask(p)
    w = decode_full(p)
    sexp = mx_shared_exponents(w, mask)
    s, mag = mx_magnitudes(w, mask, sexp)
    sk = s[mask].reshape(p.rows, p.K).astype(np.uint32)
    mk = mag[mask].reshape(p.rows, p.K).astype(np.uint32)
    hb = MX_MAG_BITS - p.t
    field = (sk << hb) | (mk >> p.t)
    lo = mk & ((1 << p.t) - 1)
    return PackedMX(p, sexp, _pack_fields(field, hb + 1, _words(p.K * (hb + 1))),
                    _pack_fields(lo, p.t, _words(p.K * p.t)))


def _decode_mx(m: PackedMX, full: bool):
    p = m.base
    hb = MX_MAG_BITS - p.t
    mask = unpack_mask(p)
    field = _unpack_fields(m.field, hb + 1, p.K).astype(np.int64)
    lo = _unpack_fields(m.lo, p.t, p.K).astype(np.int64)
    out = np.zeros((p.rows, p.cols), dtype=np.uint16)
    if full:
        out[~mask] = _unpack_fields(p.pruned, 16, p.cols - p.K).reshape(-1)
    for r in range(p.rows):
        cols_kept = np.nonzero(mask[r])[0]
        for e, c in enumerate(cols_kept):
            mag = (field[r, e] & ((1 << hb) - 1)) << p.t
            if full:
                mag |= lo[r, e]
            out[r, c] = mx_to_bf16(field[r, e] >> hb, m.sexp[r, c // MX_BLOCK], mag)
    return out


def decode_draft_mx(m: PackedMX):
    """Draft view of the shared-exponent form: leading magnitude bits only, pruned
    positions +0 (zero padding, Sec. 4.1)."""
    return _decode_mx(m, False)


def decode_full_mx(m: PackedMX):
    """Target view: all magnitude bits, pruned values merged back unchanged.  Equals the
    shared-exponent conversion of the kept values, not the original matrix (Sec. 4.2: this
    configuration trades accuracy for size)."""
    return _decode_mx(m, True)


def mx_convert(w_u16, mask):
    """The conversion stated as arithmetic on real numbers: per block, scale 2^(E - 134)
    with E the largest kept exponent; every kept finite value becomes the scale times the
    integer part of |value| / scale, sign kept.  Other entries pass through."""
    w = np.asarray(w_u16, dtype=np.uint16)
    rows, cols = w.shape
    out = w.copy()
    v = bf16_to_f64(w)
    for r in range(rows):
        for b0 in range(0, cols, MX_BLOCK):
            idx = b0 + np.nonzero(mask[r, b0:b0 + MX_BLOCK])[0]
            if idx.size == 0:
                continue
            amax = np.abs(v[r, idx]).max()
            E = max(int(math.floor(math.log2(amax))) + 127, 1) if amax > 0 else 1
            scale = math.ldexp(1.0, E - 134)
            q = np.floor(np.abs(v[r, idx]) / scale) * scale
            out[r, idx] = f64_to_bf16(np.copysign(q, v[r, idx]))
    return out


def gemv_draft_mx(m: PackedMX, x_u16):
    return gemv(decode_draft_mx(m), x_u16)


# ----------------------------------------------------------------------------
# GEMV / GEMM on reconstructed data (Sec. 4.1: ordinary FP units on bf16)
# ----------------------------------------------------------------------------
def gemv(w_u16, x_u16):
    """y = W x with W, x widened from bf16; one column; float64."""
    return bf16_to_f64(w_u16) @ bf16_to_f64(x_u16)


def gemv_draft(p: Packed, x_u16):
    """Draft GEMV: weights are the zero-padded speculation data (Sec. 4.1)."""
    return gemv(decode_draft(p), x_u16)


def gemm_verify(p: Packed, X_u16):
    """Verification GEMM (Sec. 2.2 batched verification, Sec. 4.1 full reconstruction):
    X is [ncols, n]; every column goes through the same one-column routine as plain
    decoding.  Returns [ncols, rows]."""
    w = decode_full(p)
    return np.stack([gemv(w, X_u16[c]) for c in range(X_u16.shape[0])], axis=0)


# ----------------------------------------------------------------------------
# Attention (Fig. 2_1 structure; Sec. 4.1 for which KV data each pass sees)
# ----------------------------------------------------------------------------
def attention_one(q, Kmat, Vmat):
    """softmax(q K^T / sqrt(d)) V for one query vector; q [d], K,V [T,d] float64."""
    d = q.shape[0]
    s = (Kmat @ q) / math.sqrt(d)
    s = s - s.max()
    p = np.exp(s)
    p = p / p.sum()
    return p @ Vmat


def attention(q_u16, k_u16, v_u16, n_q_heads: int, n_kv_heads: int):
    """q [n_q_heads, d] bf16; k, v [T, n_kv_heads, d] bf16 (already reconstructed for
    the pass at hand).  Grouped-query: q head h reads kv head h // (nq/nkv).
    Returns bf16 [n_q_heads, d]."""
    q = bf16_to_f64(q_u16)
    k = bf16_to_f64(k_u16)
    v = bf16_to_f64(v_u16)
    grp = n_q_heads // n_kv_heads
    out = np.zeros_like(q)
    for h in range(n_q_heads):
        out[h] = attention_one(q[h], k[:, h // grp, :], v[:, h // grp, :])
    return f64_to_bf16(out)


# ----------------------------------------------------------------------------
# Llama-3 style decoder ops; every tensor crossing an op boundary is bf16
# ----------------------------------------------------------------------------
def rmsnorm(h_u16, g_u16, eps: float):
    x = bf16_to_f64(h_u16)
    r = 1.0 / math.sqrt(float(np.mean(x * x)) + eps)
    return f64_to_bf16(x * r * bf16_to_f64(g_u16))


def rope(x_u16, pos: int, table):
    """Rotate pairs (i, i + d/2) of each head by the angle of `pos`; table is
    [max_pos, d/2, 2] cos/sin float32 (an input shared as data)."""
    x = bf16_to_f64(x_u16)
    half = x.shape[-1] // 2
    c = table[pos, :, 0].astype(np.float64)
    s = table[pos, :, 1].astype(np.float64)
    a, b = x[..., :half], x[..., half:]
    return f64_to_bf16(np.concatenate([a * c - b * s, b * c + a * s], axis=-1))


def swiglu(gate_f64, up_f64):
    g = round_bf16(gate_f64)
    u = round_bf16(up_f64)
    return f64_to_bf16(g / (1.0 + np.exp(-g)) * u)


def add_bf16(h_u16, y_f64):
    return f64_to_bf16(bf16_to_f64(h_u16) + round_bf16(y_f64))


def argmax_lowest(logits):
    return int(np.argmax(logits))  # numpy returns the first (lowest) index among maxima


# ----------------------------------------------------------------------------
# Model container and the two passes
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class KVStore:
    """Compressed cache of one layer: one Packed per committed token for K and for V
    (rows = kv heads).  Kept as lists so the oracle stays a direct transcription."""
    k: list
    v: list


class OracleModel:
    """Weights in Cassandra format + compressed KV cache + the passes of Sec. 4.1.

    shape: object with hidden, n_layers, n_q_heads, n_kv_heads, head_dim, ffn,
    vocab, rms_eps.  weights: dict as produced by synth.model_weights.  All linear
    layers including the output head are stored encoded; embedding and norm gains
    stay bf16.
    """

    def __init__(self, shape, weights, rope_tab, w_keep=600, w_t=4, kv_keep=600, kv_t=4,
                 act_norms=None, exp_mode="raw", kv_exp_mode="raw"):
        """exp_mode "raw": exponents stored as they are (also stands for the unary form, which is
        a lossless re-coding of the same data).  "mx": every linear layer in the shared-exponent
        form of Sec. 4.2; the target model is then the converted one.  kv_exp_mode: the same
        choice for the cache (Sec. 5.1 encoder: the speculation group of a new vector goes
        through the exponent compression before it is stored); with "mx" a cached vector is read
        back as its converted form by the target pass and as sign + leading magnitude bits by
        the draft pass, a block being the 32 channels of one bitmap word."""
        assert exp_mode in ("raw", "mx") and kv_exp_mode in ("raw", "mx")
        self.exp_mode, self.kv_exp_mode = exp_mode, kv_exp_mode
        self.s = shape
        self.rope_tab = rope_tab
        self.kv_keep, self.kv_t = kv_keep, kv_t
        self.embed = weights["embed"]
        self.g_final = weights["g_final"]
        an = act_norms or {}
        self.layers = []
        for li, lw in enumerate(weights["layers"]):
            enc = {}
            for name in ("wqkv", "wo", "wgu", "wd"):
                enc[name] = encode_weight(lw[name], w_keep, w_t, an.get((li, name)))
            enc["g_attn"], enc["g_ffn"] = lw["g_attn"], lw["g_ffn"]
            self.layers.append(enc)
        self.lm_head = encode_weight(weights["lm_head"], w_keep, w_t, an.get("lm_head"))
        # decoded views (the reconstruction is exact/defined; cache it for speed)
        self._dec = {}
        self.cache = [KVStore([], []) for _ in range(shape.n_layers)]

    # -- reconstruction of weights for a pass
    def W(self, layer, name, draft: bool):
        key = (layer, name, draft)
        if key not in self._dec:
            p = self.lm_head if layer is None else self.layers[layer][name]
            if self.exp_mode == "mx":
                mxp = to_mx(p)
                self._dec[key] = bf16_to_f64(decode_draft_mx(mxp) if draft else decode_full_mx(mxp))
            else:
                self._dec[key] = bf16_to_f64(decode_draft(p) if draft else decode_full(p))
        return self._dec[key]

    def cache_len(self):
        return len(self.cache[0].k)

    def _cache_kv(self, layer, draft: bool):
        st = self.cache[layer]
        if self.kv_exp_mode == "mx":
            dec = decode_draft_mx if draft else decode_full_mx
        else:
            dec = decode_draft if draft else decode_full
        if not st.k:
            z = np.zeros((0, self.s.n_kv_heads, self.s.head_dim), dtype=np.uint16)
            return z, z.copy()
        return (np.stack([dec(p) for p in st.k]), np.stack([dec(p) for p in st.v]))

    def forward(self, tokens, draft: bool, extra_kv=None):
        """Run the columns `tokens` (ids) at positions cache_len + len(extra) + c.

        draft=True : speculation data only for weights and cache (Sec. 4.1 draft
                     inference); extra_kv carries the uncompressed K/V of earlier
                     in-flight draft tokens per layer.
        draft=False: full reconstruction (Sec. 4.1 target inference); columns see the
                     cache and the exact K/V of the earlier columns of this call.
        Returns (logits [ncols, vocab] float64, new_kv per layer: list of (k, v) bf16
        [ncols, n_kv_heads, d])."""
        s = self.s
        nc = len(tokens)
        base = self.cache_len() + (0 if extra_kv is None else extra_kv[0][0].shape[0])
        h = [self.embed[int(tk)].copy() for tk in tokens]
        new_kv = []
        for li in range(s.n_layers):
            L = self.layers[li]
            ck, cv = self._cache_kv(li, draft)
            if extra_kv is not None:
                ck = np.concatenate([ck, extra_kv[li][0]], axis=0)
                cv = np.concatenate([cv, extra_kv[li][1]], axis=0)
            nk = np.zeros((nc, s.n_kv_heads, s.head_dim), dtype=np.uint16)
            nv = np.zeros_like(nk)
            for c in range(nc):
                xn = rmsnorm(h[c], L["g_attn"], s.rms_eps)
                qkv = f64_to_bf16(self.W(li, "wqkv", draft) @ bf16_to_f64(xn))
                q = qkv[: s.q_dim].reshape(s.n_q_heads, s.head_dim)
                k = qkv[s.q_dim: s.q_dim + s.kv_dim].reshape(s.n_kv_heads, s.head_dim)
                v = qkv[s.q_dim + s.kv_dim:].reshape(s.n_kv_heads, s.head_dim)
                q = rope(q, base + c, self.rope_tab)
                k = rope(k, base + c, self.rope_tab)
                nk[c], nv[c] = k, v
                kk = np.concatenate([ck, nk[: c + 1]], axis=0)
                vv = np.concatenate([cv, nv[: c + 1]], axis=0)
                o = attention(q, kk, vv, s.n_q_heads, s.n_kv_heads).reshape(-1)
                h[c] = add_bf16(h[c], self.W(li, "wo", draft) @ bf16_to_f64(o))
                xn2 = rmsnorm(h[c], L["g_ffn"], s.rms_eps)
                gu = self.W(li, "wgu", draft) @ bf16_to_f64(xn2)
                act = swiglu(gu[0::2], gu[1::2])
                h[c] = add_bf16(h[c], self.W(li, "wd", draft) @ bf16_to_f64(act))
            new_kv.append((nk, nv))
        logits = np.zeros((nc, s.vocab))
        for c in range(nc):
            xn = rmsnorm(h[c], self.g_final, s.rms_eps)
            logits[c] = self.W(None, "lm_head", draft) @ bf16_to_f64(xn)
        return logits, new_kv

    def append_kv(self, new_kv, n_cols: int):
        """Encode and append the first n_cols columns of target-computed K/V
        (Sec. 5.1 encoder: online formatting of the KV cache)."""
        for li, (nk, nv) in enumerate(new_kv):
            for c in range(n_cols):
                pk, pv = encode_kv(nk[c], self.kv_keep, self.kv_t), encode_kv(nv[c], self.kv_keep, self.kv_t)
                if self.kv_exp_mode == "mx":
                    pk, pv = to_mx(pk), to_mx(pv)
                self.cache[li].k.append(pk)
                self.cache[li].v.append(pv)

    def truncate(self, n: int):
        for st in self.cache:
            del st.k[n:], st.v[n:]


# ----------------------------------------------------------------------------
# Acceptance (Sec. 2.2, greedy rule) and the decode loops
# ----------------------------------------------------------------------------
def accept_greedy(draft, target):
    """draft: k drafted tokens; target: k+1 target tokens (target[i] is the target
    model's token after the prefix ending in draft[i-1]).  Accept the longest prefix
    on which they are identical, then emit the target's own next token.
    Returns (n_accepted, emitted tokens of length n_accepted + 1)."""
    k = len(draft)
    n = 0
    while n < k and int(draft[n]) == int(target[n]):
        n += 1
    return n, [int(x) for x in draft[:n]] + [int(target[n])]


def accept_sampling(p_target, q_draft, r):
    """Rejection-sampling acceptance (Eq. 1): n = min({i-1 : 1 <= i <= gamma, r_i > p_i/q_i} U {gamma}),
    with p_i, q_i the target / draft probability of the i-th drafted token and r_i uniform in
    [0, 1).  Inputs are the three length-gamma sequences; returns n."""
    gamma = len(r)
    cands = [gamma]
    for i in range(1, gamma + 1):
        if float(r[i - 1]) > float(p_target[i - 1]) / float(q_draft[i - 1]):
            cands.append(i - 1)
    return min(cands)


def objective_j(alpha, s_w, w_keep, w_t, s_kv, kv_keep, kv_t, b_bits=BF16_BITS):
    """Eq. 2: acceptance rate per bit read by the draft model.  w_keep, kv_keep are the kept
    fractions 1 - w_p, 1 - kv_p."""
    return alpha / (s_w * w_keep * (b_bits - w_t) + s_kv * kv_keep * (b_bits - kv_t))


def tune_grid(alpha, keeps, truncs, s_w, s_kv, kv_keep, kv_t, b_bits=BF16_BITS):
    """Grid search of Sec. 7.2.2 over the weight format: the pair with the largest J, the first
    one in row-major order among equals."""
    best, arg = -1.0, None
    for i, kp in enumerate(keeps):
        for j, t in enumerate(truncs):
            v = objective_j(alpha[i][j], s_w, kp, t, s_kv, kv_keep, kv_t, b_bits)
            if v > best:
                best, arg = v, (i, j)
    return arg


def expected_tokens_per_round(alpha: float, gamma: int) -> float:
    """Speed model of Sec. 2.2 with a per-token acceptance probability alpha (reading: the
    acceptance rate is the probability that a drafted token is accepted, independently per
    position): the i-th draft is accepted iff all of 1..i are, so a round emits
    1 + alpha + alpha^2 + ... + alpha^gamma tokens on average (the accepted drafts and the
    target's own next token)."""
    return sum(float(alpha) ** i for i in range(0, gamma + 1))


def speed_model(alpha: float, gamma: int, t_draft: float, t_verify: float, t_plain: float):
    """Sec. 2.2: a round of gamma draft passes and one verification pass costs
    gamma * t_draft + t_verify; plain decoding costs t_plain per token.  Returns
    (tokens per round, tokens per second, speedup over plain decoding)."""
    n = expected_tokens_per_round(alpha, gamma)
    rate = n / (gamma * t_draft + t_verify)
    return n, rate, rate * t_plain


def tune_measured(alpha, t_draft, t_verify, gamma: int):
    """Format search with measured pass times in place of Eq. 2's bit count (Sec. 7.2.2 searches
    the grid for the best acceptance per cost; here the cost of a format is the measured time of
    its draft and verification passes): the grid point with the most tokens per second under the
    speed model of Sec. 2.2, the first one in row-major order among equals.  alpha, t_draft,
    t_verify: [n_keep][n_trunc]."""
    best, arg = -1.0, None
    for i in range(len(alpha)):
        for j in range(len(alpha[i])):
            v = expected_tokens_per_round(alpha[i][j], gamma) / (gamma * t_draft[i][j] + t_verify[i][j])
            if v > best:
                best, arg = v, (i, j)
    return arg


def token_prob(logits, token: int) -> float:
    """Probability of `token` under the softmax of one row of logits (p_i(x), q_i(x) of Eq. 1:
    'the probability of the i-th token obtained from the model's logits')."""
    z = np.asarray(logits, dtype=np.float64)
    e = np.exp(z - z.max())
    return float(e[int(token)] / e.sum())


def spec_round_sampling(model: "OracleModel", pending: int, k: int, r):
    """One round with the acceptance rule of Eq. 1 (Sec. 2.2).  Readings where the paper is
    silent: the drafted tokens are the draft model's greedy tokens, and the token emitted after the
    n accepted drafts is the target model's greedy token at that position (Eq. 1 only defines n).
    r: k uniform numbers.  Returns (n, emitted tokens, p, q) and appends the accepted
    positions to the model's cache."""
    s = model.s
    drafts, cur, q = [], int(pending), []
    extra = [(np.zeros((0, s.n_kv_heads, s.head_dim), np.uint16),) * 2 for _ in range(s.n_layers)]
    for _ in range(k):
        lg, nkv = model.forward([cur], draft=True, extra_kv=extra)
        extra = [(np.concatenate([e[0], n[0]]), np.concatenate([e[1], n[1]])) for e, n in zip(extra, nkv)]
        cur = argmax_lowest(lg[0])
        drafts.append(cur)
        q.append(token_prob(lg[0], cur))
    vlogits, vkv = model.forward([int(pending)] + drafts, draft=False)
    p = [token_prob(vlogits[i], drafts[i]) for i in range(k)]
    n = accept_sampling(p, q, r)
    emitted = drafts[:n] + [argmax_lowest(vlogits[n])]
    model.append_kv(vkv, n + 1)
    return n, emitted, p, q


def prefill(model: OracleModel, prompt):
    """Fill the cache for prompt[:-1] with the target model; prompt[-1] stays pending."""
    if len(prompt) > 1:
        _, kv = model.forward(prompt[:-1], draft=False)
        model.append_kv(kv, len(prompt) - 1)
    return int(prompt[-1])


def plain_decode(model: OracleModel, prompt, n_new: int):
    """Autoregressive decoding with the target model (Fig. 2_3 (a))."""
    pending = prefill(model, prompt)
    out = []
    while len(out) < n_new:
        logits, kv = model.forward([pending], draft=False)
        model.append_kv(kv, 1)
        pending = argmax_lowest(logits[0])
        out.append(pending)
    return out


def spec_decode(model: OracleModel, prompt, n_new: int, k: int, stats=None):
    """Self-speculative decoding (Fig. 2_3 (b), Sec. 4.1): k draft steps on the
    speculation data, one verification pass over the pending token and the k drafts,
    greedy acceptance, commit of the accepted target K/V."""
    pending = prefill(model, prompt)
    out = []
    while len(out) < n_new:
        drafts, cur = [], pending
        extra = [(np.zeros((0, model.s.n_kv_heads, model.s.head_dim), np.uint16),) * 2
                 for _ in range(model.s.n_layers)]
        for _ in range(k):
            logits, kv = model.forward([cur], draft=True, extra_kv=extra)
            extra = [(np.concatenate([e[0], n[0]]), np.concatenate([e[1], n[1]]))
                     for e, n in zip(extra, kv)]
            cur = argmax_lowest(logits[0])
            drafts.append(cur)
        logits, kv = model.forward([pending] + drafts, draft=False)
        target = [argmax_lowest(logits[c]) for c in range(k + 1)]
        n, emitted = accept_greedy(drafts, target)
        model.append_kv(kv, n + 1)
        out.extend(emitted)
        pending = emitted[-1]
        if stats is not None:
            stats.append(n)
    return out[:n_new]
