"""Pins of the unary exponent code of the oracle (Sec. 4.2 exponent compression, Sec. 5.1
decoder): printed code words, a plain sequential scan, closed-form lengths, exhaustive search
over code assignments, and losslessness against the raw-exponent form."""
import itertools
import os

import numpy as np
import pytest

from oracle import cassandra_oracle as O
import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "unary_code_words.txt")


def _sequential(bits, numel):
    """The definition read off the code words: a value is the number of zeros before each one."""
    out, run = [], 0
    for b in bits:
        if b:
            out.append(run)
            run = 0
        else:
            run += 1
    return np.array(out[:numel], dtype=np.int64)


def test_code_words_printed_in_the_paper():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        rank, word = line.split()
        assert "".join(map(str, O.unary_encode_bits([int(rank)]))) == word


def test_every_short_stream_round_trips():
    # all rank tuples with up to 4 codes and ranks up to 5: 1 + 6 + 36 + 216 + 1296 streams
    for n in range(5):
        for ranks in itertools.product(range(6), repeat=n):
            bits = O.unary_encode_bits(ranks)
            assert len(bits) == sum(ranks) + n
            np.testing.assert_array_equal(O.unary_decode_chunked(bits, n), np.array(ranks, dtype=np.int64))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_chunked_decoder_equals_sequential_scan(seed):
    rng = np.random.Generator(np.random.Philox(seed))
    # geometric ranks with a few very long codes: runs of zeros that cross several 8-bit chunks
    ranks = rng.geometric(0.35, size=500) - 1
    ranks[rng.integers(0, 500, size=12)] = rng.integers(8, 255, size=12)
    ranks[0] = 17
    bits = O.unary_encode_bits(ranks)
    bits = np.concatenate([bits, np.zeros(19, dtype=np.uint8)])     # zero padding to a word boundary
    np.testing.assert_array_equal(O.unary_decode_chunked(bits, 500), _sequential(bits, 500))
    np.testing.assert_array_equal(O.unary_decode_chunked(bits, 500), ranks)
    np.testing.assert_array_equal(O.unary_decode_chunked(bits, 37), ranks[:37])


def test_frequency_order_minimises_the_length():
    # 4 symbols: among all 24 assignments of ranks, the frequency order gives the fewest bits
    rng = np.random.Generator(np.random.Philox(5))
    for _ in range(20):
        counts = rng.integers(0, 50, size=4)
        exps = np.repeat(np.arange(4), counts)
        exp_of_rank, rank_of_exp = O.unary_codebook(exps)
        got = int(((rank_of_exp[:4].astype(np.int64) + 1) * counts).sum())
        best = min(sum((perm[e] + 1) * counts[e] for e in range(4)) for perm in itertools.permutations(range(4)))
        assert got == best
        assert sorted(exp_of_rank.tolist()) == list(range(256)) and (exp_of_rank[rank_of_exp] == np.arange(256)).all()
    # ties go to the smaller exponent; unseen exponents follow in ascending order
    e, r = O.unary_codebook(np.array([7, 7, 3, 3, 200]))
    assert e[:4].tolist() == [3, 7, 200, 0] and r[3] == 0 and r[7] == 1 and r[200] == 2 and r[0] == 3 and r[1] == 4


@pytest.mark.parametrize("rows,cols,keep,t", [(9, 300, 600, 4), (4, 77, 250, 0), (6, 128, 1000, 7), (3, 64, 0, 4),
                                              (5, 2100, 600, 3)])
def test_unary_form_is_lossless_and_sized_in_closed_form(rows, cols, keep, t):
    W = synth.weight_matrix(rows, cols, seed=cols + t)
    W[0, : min(cols, 40)] = np.arange(min(cols, 40), dtype=np.uint16) * 0x0333 + 0x0080     # many exponents
    p = O.encode_weight(W, keep, t)
    u = O.to_unary(p)
    np.testing.assert_array_equal(O.decode_draft_unary(u), O.decode_draft(p))
    np.testing.assert_array_equal(O.decode_full_unary(u), W)
    # closed form: a row holds sum(rank + 1) bits, rounded up to words
    mask = O.unpack_mask(p)
    _, rank_of_exp = O.unary_codebook(((W[mask] >> 7) & 0xFF))
    for r in range(rows):
        bits = int((rank_of_exp[(W[r][mask[r]] >> 7) & 0xFF].astype(np.int64) + 1).sum())
        assert int(u.ue_off[r + 1] - u.ue_off[r]) == (bits + 31) // 32
    assert u.sm.shape == (rows, (p.K * (8 - t) + 31) // 32)
    x = synth.activations(cols, 1, seed=3)[0]
    np.testing.assert_array_equal(O.gemv_draft_unary(u, x), O.gemv_draft(p, x))


def test_all_exponents_and_special_values_survive():
    # every exponent 0..255 with both signs: zeros, subnormals, Inf and NaN included
    W = (np.arange(512, dtype=np.uint16).reshape(2, 256) % 256 << 7 | 0x55).astype(np.uint16)
    W[1] |= 0x8000
    p = O.encode_weight(W, 1000, 4)
    u = O.to_unary(p)
    np.testing.assert_array_equal(O.decode_full_unary(u), W)
    np.testing.assert_array_equal(O.decode_draft_unary(u), W & 0xFFF0)


def test_average_exponent_bits_on_gaussian_weights():
    """The exponents of N(0, sigma^2) weights concentrate on a few values: the unary code
    stays within a bit of their entropy (the paper reports 2.85 bits on trained models; that
    figure needs their weights and is not pinned here)."""
    W = synth.weight_matrix(64, 4096, seed=9)
    p = O.encode_weight(W, 600, 4)
    mask = O.unpack_mask(p)
    exps = (W[mask] >> 7) & 0xFF
    counts = np.bincount(exps, minlength=256).astype(np.float64)
    pr = counts[counts > 0] / counts.sum()
    entropy = float(-(pr * np.log2(pr)).sum())
    _, rank_of_exp = O.unary_codebook(exps)
    avg = float((rank_of_exp[exps].astype(np.float64) + 1).mean())
    assert entropy <= avg < entropy + 1.0
    assert avg < 4.0
