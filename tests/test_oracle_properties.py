"""Property tests of the oracle over random small shapes (hypothesis): invariants that hold for
every matrix, kept fraction and truncation (Sec. 4.1 / 4.2): exact reconstruction from both data
sets, the draft as a bit prefix of the target on kept positions and +0 elsewhere, the kept count
per row, and the same for the unary and shared-exponent forms of the speculation data."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import cassandra_oracle as O


@st.composite
def matrices(draw):
    rows = draw(st.integers(1, 6))
    cols = draw(st.integers(1, 100))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    kind = draw(st.sampled_from(["any", "normal"]))
    rng = np.random.default_rng(seed)
    if kind == "any":      # arbitrary bit patterns: zeros, subnormals, Inf and NaN included
        w = rng.integers(0, 65536, size=(rows, cols)).astype(np.uint16)
    else:
        w = O.f64_to_bf16(rng.standard_normal((rows, cols)) * np.exp2(rng.integers(-8, 3, (rows, cols)).astype(float)))
    keep = draw(st.sampled_from([0, 250, 500, 600, 999, 1000]))
    t = draw(st.integers(0, 7))
    return w, keep, t


@settings(max_examples=120, deadline=None)
@given(matrices())
def test_split_and_reconstruction_invariants(case):
    w, keep, t = case
    p = O.encode_weight(w, keep, t)
    mask = O.unpack_mask(p)
    assert (mask.sum(axis=1) == O.kept_count(w.shape[1], keep)).all()
    np.testing.assert_array_equal(O.decode_full(p), w)
    d = O.decode_draft(p)
    assert (d[~mask] == 0).all()
    np.testing.assert_array_equal(d[mask], w[mask] & np.uint16((0xFFFF << t) & 0xFFFF))
    # stream sizes follow the closed form
    bw, sw, lw, pw = O.stream_words(w.shape[1], p.K, t)
    assert p.bitmap.shape[1] == bw and p.spec.shape[1] == sw and p.lo.shape[1] == lw and p.pruned.shape[1] == pw


@settings(max_examples=60, deadline=None)
@given(matrices())
def test_unary_form_is_lossless(case):
    w, keep, t = case
    p = O.encode_weight(w, keep, t)
    u = O.to_unary(p)
    np.testing.assert_array_equal(O.decode_full_unary(u), w)
    np.testing.assert_array_equal(O.decode_draft_unary(u), O.decode_draft(p))
    # every code is its rank in zeros and a one: the stream holds exactly one one-bit per kept value
    ones = sum(int(np.unpackbits(np.ascontiguousarray(u.ue[int(u.ue_off[r]): int(u.ue_off[r + 1])].astype("<u4")).view(np.uint8)).sum())
               for r in range(p.rows))
    assert ones == p.rows * p.K


@settings(max_examples=60, deadline=None)
@given(matrices())
def test_shared_exponent_form_invariants(case):
    w, keep, t = case
    p = O.encode_weight(w, keep, t)
    mask = O.unpack_mask(p)
    m = O.to_mx(p)
    full, draft = O.decode_full_mx(m), O.decode_draft_mx(m)
    np.testing.assert_array_equal(full[~mask], w[~mask])
    assert (draft[~mask] == 0).all()
    assert ((full >> 15) == (w >> 15))[mask].all()           # signs survive
    finite = mask & (((w >> 7) & 0xFF) != 0xFF)
    blocks_finite = np.ones_like(mask)
    for r in range(w.shape[0]):                                # a block holding Inf / NaN has no numeric meaning
        for b0 in range(0, w.shape[1], 32):
            sl = slice(b0, b0 + 32)
            if (mask[r, sl] & (((w[r, sl] >> 7) & 0xFF) == 0xFF)).any():
                blocks_finite[r, sl] = False
    ok = finite & blocks_finite
    a, f, d = (np.abs(O.bf16_to_f64(x)) for x in (w, full, draft))
    assert (f[ok] <= a[ok]).all() and (d[ok] <= f[ok]).all()  # both steps drop bits, never add
    again = O.decode_full_mx(O.to_mx(O.pack(full, mask, t)))
    np.testing.assert_array_equal(again, full)                # converting twice changes nothing
