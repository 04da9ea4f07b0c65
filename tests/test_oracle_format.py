"""Pins of the oracle's format layer against what the paper and arithmetic fix.
CPU only."""
import itertools

import numpy as np
import pytest
import torch

from oracle import cassandra_oracle as O
import synth


def _golden():
    d = {}
    with open(__file__.rsplit("/", 1)[0] + "/golden/eq2_default_config.txt") as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = v
    return d


def test_golden_field_widths_and_eq2_term():
    g = _golden()
    assert int(g["bf16_sign_bits"][0]) + int(g["bf16_exponent_bits"][0]) + int(g["bf16_mantissa_bits"][0]) == O.BF16_BITS
    # exponent is half of the word (Sec. 4.2)
    assert 2 * int(g["bf16_exponent_bits"][0]) == O.BF16_BITS
    t = int(g["default_trunc_bits"][0])
    keep = 1000 - 10 * int(g["default_prune_percent"][0])
    assert O.BF16_BITS - t == int(g["draft_bits_per_kept_value"][0])
    K = O.kept_count(4096, keep)
    bw, sw, lw, pw = O.stream_words(4096, K, t)
    assert K * (O.BF16_BITS - t) == int(g["packed_spec_bits_S4096"][0])
    # Eq. 2's term differs from the packed size only through the rounding of K
    assert abs(K * (16 - t) - float(g["eq2_term_bits_S4096"][0])) < (16 - t)
    assert sw == (K * 12 + 31) // 32 and lw == (K * 4 + 31) // 32 and pw == ((4096 - K) * 16 + 31) // 32
    assert bw == 128


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-45, np.inf, -np.inf]])
    mine = O.f64_to_bf16(x.astype(np.float32).astype(np.float64))
    ref = torch.tensor(x.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(mine, ref)
    # widening is exact
    allp = np.arange(65536, dtype=np.uint16)
    ref64 = torch.tensor(allp.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = O.bf16_to_f64(allp)
    ok = np.isnan(ref64) | (ref64 == got)
    assert ok.all() and (np.isnan(ref64) == np.isnan(got)).all()


@pytest.mark.parametrize("t", range(8))
def test_exhaustive_roundtrip_all_patterns(t):
    """decode_full(encode(x)) == x for every bf16 pattern at kept and pruned positions;
    draft bits are the bit-prefix (Sec. 4.1, 4.2)."""
    pat = np.arange(65536, dtype=np.uint16).reshape(256, 256)
    w = np.repeat(pat, 2, axis=1)                  # each pattern at columns 2j and 2j+1
    mask = np.zeros(w.shape, dtype=bool)
    mask[:, 0::2] = True                           # even copy kept, odd copy pruned
    p = O.pack(w, mask, t)
    assert p.K == 256 and p.cols == 512
    np.testing.assert_array_equal(O.decode_full(p), w)
    d = O.decode_draft(p)
    himask = np.uint16((0xFFFF << t) & 0xFFFF)
    np.testing.assert_array_equal(d[:, 0::2], pat & himask)
    assert (d[:, 1::2] == 0).all()
    assert ((d[:, 0::2] ^ pat) < (1 << t)).all()   # dropped bits only


def _stream_int(words):
    v = 0
    for i, wd in enumerate(words):
        v |= int(wd) << (32 * i)
    return v


@pytest.mark.parametrize("t,keep", [(4, 600), (4, 250), (0, 1000), (7, 500), (3, 0), (5, 1000)])
def test_stream_bit_positions_by_hand(t, keep):
    """Field e of each stream sits at bit e*width of a little-endian bit stream; bitmap bit
    c of a row is bit c%32 of word c//32.  Checked with Python integers, no numpy packing."""
    cols = 77
    w = synth.normal_bf16((5, cols), 1.0, seed=3)
    p = O.encode_weight(w, keep, t)
    K = O.kept_count(cols, keep)
    assert p.K == K
    assert p.bitmap.shape[1] == 3 and p.spec.shape[1] == (K * (16 - t) + 31) // 32
    assert p.lo.shape[1] == (K * t + 31) // 32 and p.pruned.shape[1] == ((cols - K) * 16 + 31) // 32
    for r in range(5):
        bm = _stream_int(p.bitmap[r])
        kept_cols = [c for c in range(cols) if (bm >> c) & 1]
        assert len(kept_cols) == K and bm >> cols == 0
        sp, lo, pr = _stream_int(p.spec[r]), _stream_int(p.lo[r]), _stream_int(p.pruned[r])
        for e, c in enumerate(kept_cols):
            assert (sp >> (e * (16 - t))) & ((1 << (16 - t)) - 1) == int(w[r, c]) >> t
            assert (lo >> (e * t)) & ((1 << t) - 1) == int(w[r, c]) & ((1 << t) - 1)
        pruned_cols = [c for c in range(cols) if not (bm >> c) & 1]
        for u, c in enumerate(pruned_cols):
            assert (pr >> (16 * u)) & 0xFFFF == int(w[r, c])
        # padding bits are zero
        assert sp >> (K * (16 - t)) == 0 and lo >> (K * t) == 0 and pr >> ((cols - K) * 16) == 0


def test_kept_count_formula():
    assert O.kept_count(4096, 600) == 2458
    assert O.kept_count(4096, 250) == 1024
    assert O.kept_count(128, 600) == 77
    assert O.kept_count(128, 1000) == 128
    assert O.kept_count(128, 0) == 0
    assert O.kept_count(14336, 600) == 8602


def _brute_select(scores, k):
    g = len(scores)
    best = None
    for sub in itertools.combinations(range(g), k):
        key = (sum(int(scores[i]) for i in sub), tuple(-i for i in sub))
        # maximise the sum; among equal sums prefer the lexicographically smallest index tuple
        if best is None or key > best[0]:
            best = (key, sub)
    return set(best[1])


@pytest.mark.parametrize("seed", range(6))
def test_selection_brute_force_small_groups(seed):
    rng = np.random.default_rng(seed)
    g = int(rng.integers(5, 11))
    k = int(rng.integers(0, g + 1))
    scores = rng.integers(0, 4, size=(7, g)).astype(np.uint32)   # many ties
    mask = O.select_topk(scores, k)
    for r in range(7):
        assert set(np.nonzero(mask[r])[0]) == (_brute_select(scores[r], k) if k else set())


def test_selection_weights_activation_aware_brute_force():
    """score = |w| * a_j: brute force with real-valued products on a tiny matrix."""
    w = synth.normal_bf16((6, 9), 1.0, seed=11)
    a = synth.act_norm(9, seed=5)
    bits = O.weight_scores(w, a)
    prod = np.abs(synth.bf16_bits_to_f32(w)) * a[None, :]
    np.testing.assert_array_equal(bits.view(np.float32), prod.astype(np.float32))
    mask = O.select_topk(bits, 4)
    for r in range(6):
        # non-negative floats order like their bit patterns
        assert set(np.nonzero(mask[r])[0]) == _brute_select(bits[r], 4)
        assert prod[r][mask[r]].min() >= prod[r][~mask[r]].max()


def test_selection_magnitude_matches_library_sort():
    w = synth.weight_matrix(64, 512, seed=2)
    K = O.kept_count(512, 600)
    mask = O.select_topk(O.weight_scores(w, None), K)
    assert (mask.sum(axis=1) == K).all()
    mag = np.abs(synth.bf16_bits_to_f32(w).astype(np.float64))
    for r in range(64):
        thr = np.sort(mag[r])[::-1][K - 1]
        assert (mag[r][mask[r]] >= thr).all() and (mag[r][~mask[r]] <= thr).all()
        ties = np.nonzero(mag[r] == thr)[0]
        kept_ties = [i for i in ties if mask[r, i]]
        # ties go to the lower index
        assert kept_ties == list(ties[: len(kept_ties)])


def test_selection_kv_is_magnitude_per_vector_with_outlier_channels():
    k = synth.kv_tensor(16, 2, 128, seed=4, outlier_channels=4)
    p = O.encode_kv(k.reshape(-1, 128), 600, 4)
    assert p.K == 77
    mask = O.unpack_mask(p)
    mag = np.abs(synth.bf16_bits_to_f32(k.reshape(-1, 128)))
    for r in range(mask.shape[0]):
        assert mag[r][mask[r]].min() >= mag[r][~mask[r]].max()


def test_nan_inf_patterns_have_total_order_and_roundtrip():
    w = np.array([[0x7FC0, 0x7F80, 0xFF80, 0x0000, 0x8000, 0x0001, 0x7F7F, 0xFFFF]], dtype=np.uint16)
    p = O.encode_weight(w, 500, 4)
    np.testing.assert_array_equal(O.decode_full(p), w)
    assert set(np.nonzero(O.unpack_mask(p)[0])[0]) == {7, 0, 1, 2}   # largest 15-bit magnitudes; ties lower index
