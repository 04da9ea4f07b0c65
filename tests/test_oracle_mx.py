"""Pins of the shared-exponent (MX) part of the oracle (Sec. 4.2 exponent compression, first
approach; Sec. 5.1 decoder #N) against things other than itself: a hand-worked block, the
conversion restated as real-number arithmetic, the lossless special case, the error bound,
idempotence, the exact value of every (exponent, magnitude) pair, and closed-form sizes."""
import math
import os

import numpy as np
import pytest

from oracle import cassandra_oracle as O
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "mx_block_example.txt")


def _wide_matrix(rows, cols, seed, spread=12):
    """bf16 matrix whose exponents spread over `spread` binades, plus zeros and subnormals."""
    rng = np.random.default_rng(seed)
    v = rng.standard_normal((rows, cols)) * np.exp2(rng.integers(-spread, 1, (rows, cols)).astype(np.float64))
    w = O.f64_to_bf16(v)
    w[rng.random((rows, cols)) < 0.02] = 0x0000
    w[rng.random((rows, cols)) < 0.02] = 0x8000
    sub = rng.random((rows, cols)) < 0.02
    w[sub] = rng.integers(1, 0x80, sub.sum()).astype(np.uint16) | (rng.integers(0, 2, sub.sum()).astype(np.uint16) << 15)
    return w


def test_hand_worked_block():
    rows = [l.split() for l in open(GOLD) if l.strip() and not l.startswith("#")]
    w = np.array([[int(r[0], 16) for r in rows]], dtype=np.uint16)
    mask = np.ones_like(w, dtype=bool)
    sexp = O.mx_shared_exponents(w, mask)
    assert sexp.tolist() == [[128]]
    s, mag = O.mx_magnitudes(w, mask, sexp)
    assert s[0].tolist() == [int(r[1]) for r in rows]
    assert mag[0].tolist() == [int(r[2], 16) for r in rows]
    m = O.to_mx(O.pack(w, mask, 4))
    assert O.decode_full_mx(m)[0].tolist() == [int(r[3], 16) for r in rows]
    assert O._unpack_fields(m.field, 5, len(rows))[0].tolist() == [int(r[4], 16) for r in rows]
    assert O.decode_draft_mx(m)[0].tolist() == [int(r[5], 16) for r in rows]


@pytest.mark.parametrize("rows,cols,keep,t", [(6, 96, 600, 4), (5, 75, 500, 0), (4, 130, 700, 7), (3, 33, 1000, 3),
                                              (4, 64, 250, 1)])
def test_bit_route_equals_real_arithmetic(rows, cols, keep, t):
    w = _wide_matrix(rows, cols, seed=rows * 1000 + cols)
    p = O.encode_weight(w, keep, t)
    mask = O.unpack_mask(p)
    np.testing.assert_array_equal(O.decode_full_mx(O.to_mx(p)), O.mx_convert(w, mask))


def test_every_exponent_magnitude_pair_is_its_real_value():
    for E in list(range(1, 20)) + [100, 127, 128, 200, 254, 255]:
        for mag in range(256):
            for sign in (0, 1):
                word = O.mx_to_bf16(sign, E, mag)
                if E == 255 and mag >= 128:
                    continue        # all-ones exponent field: not a number in bf16
                want = (-1.0) ** sign * mag * 2.0 ** (E - 134)
                got = float(O.bf16_to_f64(np.array([word], dtype=np.uint16))[0])
                assert got == want and (word >> 15) == sign, (E, mag, sign, hex(word))


def test_blocks_of_one_exponent_are_lossless():
    rng = np.random.default_rng(2)
    rows, cols = 5, 128
    exps = rng.integers(1, 255, (rows, cols // 32)).repeat(32, axis=1)
    w = ((rng.integers(0, 2, (rows, cols)) << 15) | (exps << 7) | rng.integers(0, 128, (rows, cols))).astype(np.uint16)
    for t in (0, 4):
        p = O.encode_weight(w, 600, t)
        np.testing.assert_array_equal(O.decode_full_mx(O.to_mx(p)), w)


@pytest.mark.parametrize("t", [0, 2, 4, 7])
def test_error_bound_direction_and_block_maximum(t):
    w = _wide_matrix(8, 160, seed=9)
    p = O.encode_weight(w, 600, t)
    mask = O.unpack_mask(p)
    m = O.to_mx(p)
    full, draft = O.decode_full_mx(m), O.decode_draft_mx(m)
    np.testing.assert_array_equal(full[~mask], w[~mask])        # pruned values untouched
    assert (draft[~mask] == 0).all()
    ulp = np.exp2(np.repeat(m.sexp.astype(np.float64), 32, axis=1)[:, :160] - 134.0)
    a, f, d = (np.abs(O.bf16_to_f64(x)) for x in (w, full, draft))
    assert (f[mask] <= a[mask]).all() and (a[mask] - f[mask] < ulp[mask]).all()
    assert (d[mask] <= f[mask]).all() and (f[mask] - d[mask] < ulp[mask] * 2 ** t).all()
    assert ((full >> 15) == (w >> 15))[mask].all() and ((draft >> 15) == (w >> 15))[mask].all()
    if t == 0:
        np.testing.assert_array_equal(draft[mask], full[mask])
    # the largest kept magnitude of every block survives bit for bit
    for r in range(8):
        for b in range(5):
            idx = 32 * b + np.nonzero(mask[r, 32 * b: 32 * b + 32])[0]
            if idx.size:
                j = idx[np.argmax(a[r, idx])]
                assert full[r, j] == w[r, j]


def test_conversion_is_idempotent():
    w = _wide_matrix(6, 96, seed=4)
    p = O.encode_weight(w, 600, 4)
    once = O.decode_full_mx(O.to_mx(p))
    again = O.decode_full_mx(O.to_mx(O.pack(once, O.unpack_mask(p), 4)))
    np.testing.assert_array_equal(once, again)


def test_stream_sizes_closed_form():
    for cols, keep, t in [(4096, 600, 4), (300, 500, 0), (64, 1000, 7)]:
        w = synth.weight_matrix(3, cols, seed=cols)
        m = O.to_mx(O.encode_weight(w, keep, t))
        K = O.kept_count(cols, keep)
        assert m.sexp.shape == (3, math.ceil(cols / 32)) and m.sexp.dtype == np.uint8
        assert m.field.shape == (3, math.ceil(K * (9 - t) / 32))
        assert m.lo.shape == (3, math.ceil(K * t / 32))


def test_all_ones_exponent_as_block_maximum_keeps_its_bits():
    w = np.array([[0x7F80, 0x3F80, 0xFFC1, 0x0001] + [0] * 28], dtype=np.uint16)   # +inf, 1.0, a NaN, a subnormal
    mask = np.zeros((1, 32), dtype=bool); mask[0, :4] = True
    full = O.decode_full_mx(O.to_mx(O.pack(w, mask, 4)))
    assert full[0, 0] == 0x7F80 and full[0, 2] == 0xFFC1 and full[0, 1] == 0x0000 and full[0, 3] == 0x0000


def test_draft_gemv_reduces_to_the_raw_form_when_nothing_is_lost():
    rng = np.random.default_rng(6)
    exps = rng.integers(100, 140, (4, 3)).repeat(32, axis=1)
    w = ((rng.integers(0, 2, (4, 96)) << 15) | (exps << 7) | (rng.integers(0, 8, (4, 96)) << 4)).astype(np.uint16)
    x = synth.activations(96, 1, seed=1)[0]
    p = O.encode_weight(w, 600, 4)          # the low four mantissa bits are zero: truncation drops nothing
    np.testing.assert_array_equal(O.gemv_draft_mx(O.to_mx(p), x), O.gemv_draft(p, x))


def test_subnormals_share_the_smallest_exponent_without_loss():
    """Values with exponent field 0 and 1 have the same scale (2^-133 per significand unit): a
    block of them converts without loss."""
    w = np.array([[0x0080, 0x0040, 0x0001, 0x80FF, 0x007F, 0x8000] + [0] * 26], dtype=np.uint16)
    mask = np.zeros((1, 32), dtype=bool); mask[0, :6] = True
    m = O.to_mx(O.pack(w, mask, 0))
    assert m.sexp[0, 0] == 1
    np.testing.assert_array_equal(O.decode_full_mx(m), w)
    np.testing.assert_array_equal(O.decode_full_mx(m), O.mx_convert(w, mask))


def test_only_kept_values_set_the_shared_exponent():
    """Selection by activation-weighted score can prune a value larger than the kept ones of
    its block (Sec. 4.2 weight pruning); it must not raise the block's exponent."""
    rng = np.random.default_rng(8)
    w = ((rng.integers(0, 2, (2, 64)) << 15) | (120 << 7) | rng.integers(0, 128, (2, 64))).astype(np.uint16)
    mask = np.ones((2, 64), dtype=bool)
    w[:, 5] = 0x4E00; mask[:, 5] = False       # a large pruned value in block 0
    w[:, 40] = 0x7F00; mask[:, 40] = False     # and in block 1
    m = O.to_mx(O.pack(w, mask, 4))
    assert (m.sexp == 120).all()
    np.testing.assert_array_equal(O.decode_full_mx(m), w)


def test_model_in_shared_exponent_mode_reduces_to_the_raw_mode_when_blocks_have_one_exponent():
    """The shared-exponent mode of the oracle's model (Sec. 4.2, the MX approach: the converted
    matrices are the weights) must give the raw mode's logits, draft and target, bit for bit when
    no block loses anything: every 32-column block of every row holds a single exponent."""
    shape = synth.TINY
    weights = synth.model_weights(shape, seed=4)
    rng = np.random.default_rng(8)

    def one_exponent_per_block(w):
        rows, cols = w.shape
        nb = (cols + 31) // 32
        exps = rng.integers(118, 123, (rows, nb)).repeat(32, axis=1)[:, :cols].astype(np.uint16)
        return ((w & 0x807F) | (exps << 7)).astype(np.uint16)

    for lw in weights["layers"]:
        for name in ("wqkv", "wo", "wgu", "wd"):
            lw[name] = one_exponent_per_block(lw[name])
    weights["lm_head"] = one_exponent_per_block(weights["lm_head"])
    tab = synth.rope_table(32, shape.head_dim, shape.rope_theta)
    raw = O.OracleModel(shape, weights, tab, w_keep=600, w_t=4, exp_mode="raw")
    mx = O.OracleModel(shape, weights, tab, w_keep=600, w_t=4, exp_mode="mx")
    toks = synth.token_ids(3, shape.vocab, seed=2)
    for draft in (False, True):
        a, _ = raw.forward(toks, draft=draft)
        b, _ = mx.forward(toks, draft=draft)
        np.testing.assert_array_equal(a, b)
    # ... and differs from it on ordinary weights (the mode is really switched on)
    weights2 = synth.model_weights(shape, seed=4)
    a, _ = O.OracleModel(shape, weights2, tab, exp_mode="raw").forward(toks, draft=False)
    b, _ = O.OracleModel(shape, weights2, tab, exp_mode="mx").forward(toks, draft=False)
    assert np.abs(a - b).max() > 0


def test_cache_in_shared_exponent_mode_against_real_arithmetic_and_the_raw_mode():
    """The oracle model's cache with kv_exp_mode="mx" (Sec. 5.1 encoder: exponent compression of
    the speculation group before storing): what the target pass reads back is, for a kept
    value, sign * floor(significand * 2^(e - E)) * 2^(E - 134) with E the largest exponent among
    the kept values of its 32-channel block, restated here in real arithmetic; unselected
    values come back as they went in; vectors whose blocks hold one exponent come back
    unchanged, as in the raw mode."""
    shape = synth.TINY
    weights = synth.model_weights(shape, seed=4)
    tab = synth.rope_table(32, shape.head_dim, shape.rope_theta)
    keep, t = 600, 4
    mx = O.OracleModel(shape, weights, tab, kv_keep=keep, kv_t=t, kv_exp_mode="mx")
    raw = O.OracleModel(shape, weights, tab, kv_keep=keep, kv_t=t, kv_exp_mode="raw")
    rng = np.random.default_rng(3)
    ncols, H, D = 3, shape.n_kv_heads, shape.head_dim
    wide = O.f64_to_bf16(rng.standard_normal((ncols, H, D)) * np.exp2(rng.integers(-6, 1, (ncols, H, D)).astype(float)))
    exps = rng.integers(110, 130, (ncols, H, D // 32)).repeat(32, axis=2)
    flat = ((rng.integers(0, 2, (ncols, H, D)) << 15) | (exps << 7) | rng.integers(0, 128, (ncols, H, D))).astype(np.uint16)
    new_kv = [(wide, flat) for _ in range(shape.n_layers)]
    mx.append_kv(new_kv, ncols)
    raw.append_kv(new_kv, ncols)
    K_mx, V_mx = mx._cache_kv(0, draft=False)
    K_raw, V_raw = raw._cache_kv(0, draft=False)
    np.testing.assert_array_equal(V_mx, flat)            # one exponent per block: nothing is lost
    np.testing.assert_array_equal(V_raw, flat)
    np.testing.assert_array_equal(K_raw, wide)           # the raw mode is lossless for any vector
    # K with mixed exponents: every value against the conversion in real arithmetic
    for c in range(ncols):
        for h in range(H):
            v = wide[c, h]
            mask = O.unpack_mask(O.encode_kv(v[None, :], keep, t))[0]
            e = np.maximum((v >> 7) & 0xFF, 1).astype(int)
            sig = ((v & 0x7F) | np.where(((v >> 7) & 0xFF) != 0, 0x80, 0)).astype(int)
            for b in range(D // 32):
                sl = slice(32 * b, 32 * b + 32)
                kept = mask[sl]
                if not kept.any():
                    continue
                E = e[sl][kept].max()
                want = np.where(v[sl] >> 15, -1.0, 1.0) * np.floor(sig[sl] * np.exp2((e[sl] - E).astype(float))) * 2.0 ** (E - 134)
                got = O.bf16_to_f64(K_mx[c, h, sl])
                np.testing.assert_array_equal(got[kept], want[kept])
                np.testing.assert_array_equal(K_mx[c, h, sl][~kept], v[sl][~kept])
    # the draft pass sees sign + leading magnitude bits of the kept values and zeros elsewhere
    K_d, _ = mx._cache_kv(0, draft=True)
    assert (np.abs(O.bf16_to_f64(K_d)) <= np.abs(O.bf16_to_f64(K_mx))).all()
    assert (K_d[~np.stack([[O.unpack_mask(O.encode_kv(wide[c, h][None, :], keep, t))[0] for h in range(H)] for c in range(ncols)])] == 0).all()
