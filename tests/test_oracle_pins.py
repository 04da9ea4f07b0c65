"""Pins of the oracle's small decoder helpers and of its forward composition against things
that are not the oracle: hand-worked bf16 roundings, tie cases, Eq. 2 worked by hand from the
figures the paper states in its text, and a separately written float64 Llama block made of
library operations (Fig. 2_1 structure).  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import cassandra_oracle as O
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bits(x):
    return int(O.f64_to_bf16(np.array([x]))[0])


# ---------------------------------------------------------------------------------------------
# residual add: the addend is rounded to bf16 first, then the sum
# ---------------------------------------------------------------------------------------------
def test_add_bf16_rounds_the_addend_before_the_sum_hand_worked():
    """Values chosen so that other readings of the residual add give different bits.
    bf16 has 8 significand bits: next to 1.0 the spacing is 2^-7, so 1 + 2^-8 is a tie."""
    one = np.array([0x3F80], dtype=np.uint16)
    # y = 2^-8 + 2^-16 rounds to 2^-8 (a tie, to the even significand); 1 + 2^-8 is a tie again and
    # goes to the even 1.0.  Adding the unrounded y gives 1 + 2^-8 + 2^-16, above the tie: 0x3F81.
    y = np.array([2.0 ** -8 + 2.0 ** -16])
    assert int(O.add_bf16(one, y)[0]) == 0x3F80
    assert _bits(1.0 + y[0]) == 0x3F81
    # y = 2^-8 - 2^-17 is a tie between 2^-8 - 2^-16 (odd significand) and 2^-8 (even): it rounds
    # to 2^-8 and the sum to 1.0; the unrounded sum is below the tie and gives 1.0 as well
    y2 = np.array([2.0 ** -8 - 2.0 ** -17])
    assert int(O.add_bf16(one, y2)[0]) == 0x3F80 == _bits(1.0 + y2[0])
    # above the tie either way
    assert int(O.add_bf16(one, np.array([2.0 ** -8 + 2.0 ** -9 - 2.0 ** -18]))[0]) == 0x3F81
    # an exact sum needs no second rounding: 2 + 0.5
    assert int(O.add_bf16(np.array([0x4000], dtype=np.uint16), np.array([0.5]))[0]) == 0x4020
    # the sum is rounded to nearest even, not truncated: 256 + 1.5 = 257.5 (spacing 2) -> 258
    h256 = O.f64_to_bf16(np.array([256.0]))
    assert int(O.add_bf16(h256, np.array([1.5]))[0]) == _bits(258.0)
    assert int(O.add_bf16(h256, np.array([0.99]))[0]) == _bits(256.0)
    # the addend is rounded, not truncated: 0.999 rounds to 1.0 (it would truncate to 0.99609375);
    # 258 + 1.0 = 259 is a tie and goes to the even significand, 260; 258.996 would go to 258
    h258 = O.f64_to_bf16(np.array([258.0]))
    assert int(O.add_bf16(h258, np.array([0.999]))[0]) == _bits(260.0)


def test_add_bf16_vector_and_sign():
    h = O.f64_to_bf16(np.array([1.0, -1.0, 0.0, -0.0]))
    y = np.array([-(2.0 ** -8 + 2.0 ** -16), 2.0 ** -8 + 2.0 ** -16, 1e-3, 0.0])
    got = O.add_bf16(h, y)
    # 1 - 2^-8: spacing below 1 is 2^-8, so the sum is exact: 0x3F7F; mirrored for -1
    assert [int(v) for v in got[:2]] == [0x3F7F, 0xBF7F]
    assert int(got[2]) == _bits(float(O.round_bf16(np.array([1e-3]))[0]))
    assert int(got[3]) == 0x0000   # -0 + +0 = +0 in round-to-nearest


# ---------------------------------------------------------------------------------------------
# greedy token: lowest index among the maxima
# ---------------------------------------------------------------------------------------------
def test_argmax_lowest_takes_the_lowest_index_among_tied_maxima():
    assert O.argmax_lowest(np.array([1.0, 3.0, 3.0, 2.0, 3.0])) == 1
    assert O.argmax_lowest(np.array([5.0, 5.0])) == 0
    assert O.argmax_lowest(np.array([-2.0, -1.0, -1.0])) == 1
    assert O.argmax_lowest(np.array([0.0, -0.0, 0.0])) == 0         # +0 and -0 compare equal
    assert O.argmax_lowest(np.array([-np.inf, -np.inf])) == 0
    x = np.full(1000, 0.25)
    x[[17, 400, 999]] = 0.5
    assert O.argmax_lowest(x) == 17
    assert O.argmax_lowest(x[::-1]) == 0                            # 999 -> index 0 after the flip


# ---------------------------------------------------------------------------------------------
# Eq. 2 and the grid search of Sec. 7.2.2, worked by hand
# ---------------------------------------------------------------------------------------------
def _golden():
    out = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "eq2_default_config.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            out[k] = [float(x) for x in v]
    return out


def test_objective_j_closed_forms():
    g = _golden()
    keep = 1.0 - g["default_prune_percent"][0] / 100.0
    t = int(g["default_trunc_bits"][0])
    # the weight term alone, S_w = 4096, default configuration: 4096 * 0.6 * 12 bits (golden file)
    assert abs(1.0 / O.objective_j(1.0, 4096.0, keep, t, 0.0, keep, t) - g["eq2_term_bits_S4096"][0]) < 1e-9
    assert 16 - t == g["draft_bits_per_kept_value"][0]
    # both terms, numbers worked by hand: S_w = 1000, keep 0.5, t = 2 -> 1000 * 0.5 * 14 = 7000;
    # S_kv = 200, keep 0.25, t = 4 -> 200 * 0.25 * 12 = 600; alpha = 0.76 -> J = 0.76 / 7600 = 1e-4
    assert abs(O.objective_j(0.76, 1000.0, 0.5, 2, 200.0, 0.25, 4) - 1e-4) < 1e-18
    # a transposed operand (weight parameters applied to the cache term) gives 0.76 / (1000*.25*12 + 200*.5*14)
    assert abs(O.objective_j(0.76, 1000.0, 0.5, 2, 200.0, 0.25, 4) - 0.76 / 4400.0) > 1e-5
    # nothing pruned, nothing truncated: every value costs B bits
    assert abs(1.0 / O.objective_j(1.0, 10.0, 1.0, 0, 6.0, 1.0, 0) - 16 * 16.0) < 1e-12
    assert abs(1.0 / O.objective_j(1.0, 10.0, 1.0, 0, 6.0, 1.0, 0, b_bits=8) - 16 * 8.0) < 1e-12
    # linear in alpha, inverse in the sizes
    a = O.objective_j(0.5, 4096.0, 0.6, 4, 100.0, 0.5, 2)
    assert abs(2 * a - O.objective_j(1.0, 4096.0, 0.6, 4, 100.0, 0.5, 2)) < 1e-18
    assert abs(2 * a - O.objective_j(0.5, 2048.0, 0.6, 4, 50.0, 0.5, 2)) < 1e-18


def test_tune_grid_hand_worked():
    g = _golden()
    keeps = [1.0 - p / 100.0 for p in g["grid_prune_percent"]]      # 0.7, 0.6, 0.5, 0.4
    truncs = [int(t) for t in g["grid_trunc_bits"]]                 # 0 .. 5
    assert keeps == [0.7, 0.6, 0.5, 0.4] and truncs == [0, 1, 2, 3, 4, 5]
    # constant acceptance: the smallest draft wins = last row, last column
    alpha = np.full((4, 6), 0.8)
    assert O.tune_grid(alpha, keeps, truncs, 1e6, 0.0, 0.6, 4) == (3, 5)
    # acceptance proportional to the bits read: every J equal -> the first pair in row-major order
    alpha = np.array([[kp * (16 - t) for t in truncs] for kp in keeps]) / 16.0
    assert O.tune_grid(alpha, keeps, truncs, 1.0, 0.0, 0.6, 4) == (0, 0)
    # one pair made slightly better than proportional wins, wherever it sits
    alpha[1, 4] *= 1.001
    assert O.tune_grid(alpha, keeps, truncs, 1.0, 0.0, 0.6, 4) == (1, 4)
    # a large fixed cache term makes the weight format irrelevant: the largest alpha wins
    alpha = np.full((4, 6), 0.5)
    alpha[2, 1] = 0.9
    assert O.tune_grid(alpha, keeps, truncs, 1.0, 1e9, 0.6, 4) == (2, 1)
    # hand numbers: S_w = 100, no cache.  (keep .7, t 0): 100*.7*16 = 1120 bits, alpha .9 -> 8.036e-4
    #                                     (keep .4, t 5): 100*.4*11 = 440 bits, alpha .3 -> 6.818e-4
    alpha = np.full((4, 6), 1e-9)
    alpha[0, 0], alpha[3, 5] = 0.9, 0.3
    assert O.tune_grid(alpha, keeps, truncs, 100.0, 0.0, 0.6, 4) == (0, 0)
    alpha[3, 5] = 0.36                                              # 0.36 / 440 = 8.18e-4 > 8.036e-4
    assert O.tune_grid(alpha, keeps, truncs, 100.0, 0.0, 0.6, 4) == (3, 5)


# ---------------------------------------------------------------------------------------------
# forward composition against a separately written float64 decoder made of library operations
# ---------------------------------------------------------------------------------------------
def _t64(u16):
    return torch.tensor(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).to(torch.float64)


def _rb(x):
    """bf16 rounding of a float64 tensor at an operation boundary (through float32, both RNE)."""
    return x.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _library_decoder(shape, w, rope_tab, tokens, past_k=None, past_v=None):
    """Llama-3 block structure (Fig. 2_1) on dense bf16 weights: RMSNorm -> qkv -> rotary ->
    grouped-query causal attention -> output projection -> residual -> RMSNorm -> SwiGLU ->
    residual; final norm and output head.  All columns at once, library kernels in float64,
    bf16 rounding wherever a tensor passes from one operation to the next.
    past_k / past_v: per layer [T0, n_kv, d] float64 (already what the pass may see)."""
    F = torch.nn.functional
    n = len(tokens)
    H, d, nq, nkv = shape.hidden, shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    T0 = 0 if past_k is None else past_k[0].shape[0]
    h = _t64(w["embed"])[torch.tensor([int(t) for t in tokens])]                      # [n, H]
    cs = torch.tensor(rope_tab[T0:T0 + n].astype(np.float64))                         # [n, d/2, 2]
    rot = torch.complex(cs[..., 0], cs[..., 1])[:, None, :]                           # e^{i pos theta_j}
    ks, vs = [], []
    for li, L in enumerate(w["layers"]):
        xn = _rb(F.rms_norm(h, (H,), _t64(L["g_attn"]), eps=shape.rms_eps))
        qkv = _rb(xn @ _t64(L["wqkv"]).T)
        q = qkv[:, : nq * d].reshape(n, nq, d)
        k = qkv[:, nq * d: (nq + nkv) * d].reshape(n, nkv, d)
        v = qkv[:, (nq + nkv) * d:].reshape(n, nkv, d)

        def rotate(x):   # channel j pairs with j + d/2; the pair is one complex number
            z = torch.complex(x[..., : d // 2], x[..., d // 2:]) * rot
            return _rb(torch.cat([z.real, z.imag], dim=-1))
        q, k = rotate(q), rotate(k)
        ks.append(k); vs.append(v)
        kk = k if past_k is None else torch.cat([past_k[li], k], dim=0)
        vv = v if past_v is None else torch.cat([past_v[li], v], dim=0)
        # query head h reads kv head h // (nq / nkv); column c sees the past and columns 0..c
        kq = kk.permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)                   # [nq, T, d]
        vq = vv.permute(1, 0, 2).repeat_interleave(nq // nkv, dim=0)
        mask = torch.ones(n, T0 + n, dtype=torch.bool).tril(diagonal=T0)
        o = _rb(F.scaled_dot_product_attention(q.permute(1, 0, 2), kq, vq, attn_mask=mask))   # [nq, n, d]
        o = o.permute(1, 0, 2).reshape(n, nq * d)
        h = _rb(h + _rb(o @ _t64(L["wo"]).T))
        xn = _rb(F.rms_norm(h, (H,), _t64(L["g_ffn"]), eps=shape.rms_eps))
        gu = _rb(xn @ _t64(L["wgu"]).T)
        act = _rb(F.silu(gu[:, 0::2]) * gu[:, 1::2])
        h = _rb(h + _rb(act @ _t64(L["wd"]).T))
    xn = _rb(F.rms_norm(h, (H,), _t64(w["g_final"]), eps=shape.rms_eps))
    return (xn @ _t64(w["lm_head"]).T).numpy(), ks, vs


@pytest.mark.parametrize("keep,t", [(1000, 0), (600, 4)])
def test_target_forward_equals_library_decoder_on_the_original_weights(keep, t):
    """The target pass reconstructs every weight exactly (Sec. 4.1), so whatever the format its
    logits are those of the dense model: checked against the library decoder, 4 columns, causal."""
    shape = synth.TINY
    w = synth.model_weights(shape, seed=3)
    tab = synth.rope_table(64, shape.head_dim, shape.rope_theta)
    m = O.OracleModel(shape, w, tab, w_keep=keep, w_t=t, kv_keep=keep, kv_t=t)
    tokens = synth.token_ids(4, shape.vocab, seed=8)
    logits, kv = m.forward(tokens, draft=False)
    ref, ks, vs = _library_decoder(shape, w, tab, tokens)
    scale = np.abs(ref).max()
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-9 * scale)
    for li in range(shape.n_layers):
        np.testing.assert_array_equal(O.bf16_to_f64(kv[li][0]), ks[li].numpy())
        np.testing.assert_array_equal(O.bf16_to_f64(kv[li][1]), vs[li].numpy())
    # second call on top of a committed cache: positions continue, the cache is read back exactly
    m.append_kv(kv, 4)
    more = synth.token_ids(2, shape.vocab, seed=9)
    logits2, _ = m.forward(more, draft=False)
    ref2, _, _ = _library_decoder(shape, w, tab, more, ks, vs)
    np.testing.assert_allclose(logits2, ref2, rtol=0, atol=1e-9 * scale)
    if keep == 1000 and t == 0:
        # draft == target when nothing is pruned or truncated
        logits3, _ = m.forward(more, draft=True)
        np.testing.assert_allclose(logits3, ref2, rtol=0, atol=1e-9 * scale)


def test_draft_forward_equals_library_decoder_on_the_zero_padded_weights_and_cache():
    """The draft pass (Sec. 4.1) is the same decoder run on the zero-padded speculation data:
    weights = decode_draft of every matrix, cache = decode_draft of the committed K/V, in-flight
    vectors uncompressed."""
    shape = synth.TINY
    w = synth.model_weights(shape, seed=4)
    tab = synth.rope_table(64, shape.head_dim, shape.rope_theta)
    m = O.OracleModel(shape, w, tab, w_keep=600, w_t=4, kv_keep=600, kv_t=4)
    prompt = synth.token_ids(5, shape.vocab, seed=10)
    _, kv = m.forward(prompt, draft=False)
    m.append_kv(kv, 5)
    wd = {"embed": w["embed"], "g_final": w["g_final"], "lm_head": O.decode_draft(m.lm_head),
          "layers": [{n: (O.decode_draft(L[n]) if n.startswith("w") else L[n]) for n in L} for L in m.layers]}
    past_k = [_t64(np.stack([O.decode_draft(p) for p in st.k])) for st in m.cache]
    past_v = [_t64(np.stack([O.decode_draft(p) for p in st.v])) for st in m.cache]
    tok = [7]
    logits, kv1 = m.forward(tok, draft=True, extra_kv=[(np.zeros((0, shape.n_kv_heads, 128), np.uint16),) * 2
                                                        for _ in range(shape.n_layers)])
    ref, ks, vs = _library_decoder(shape, wd, tab, tok, past_k, past_v)
    scale = np.abs(ref).max()
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-9 * scale)
    # second draft step: the first step's K/V ride along uncompressed
    logits, _ = m.forward([11], draft=True, extra_kv=kv1)
    pk = [torch.cat([a, b], dim=0) for a, b in zip(past_k, ks)]
    pv = [torch.cat([a, b], dim=0) for a, b in zip(past_v, vs)]
    ref, _, _ = _library_decoder(shape, wd, tab, [11], pk, pv)
    np.testing.assert_allclose(logits, ref, rtol=0, atol=1e-9 * scale)


# ---- speed model of Sec. 2.2, the format search on measured times, softmax probabilities of Eq. 1
def test_expected_tokens_per_round_closed_forms_and_enumeration():
    import itertools
    # closed form of the geometric series, and the two ends
    for gamma in range(0, 9):
        assert O.expected_tokens_per_round(0.0, gamma) == 1.0
        assert O.expected_tokens_per_round(1.0, gamma) == gamma + 1
        for a in (0.1, 0.5, 0.8, 0.97):
            assert abs(O.expected_tokens_per_round(a, gamma) - (1 - a ** (gamma + 1)) / (1 - a)) < 1e-12
    assert abs(O.expected_tokens_per_round(0.5, 3) - 1.875) < 1e-15          # 1 + 1/2 + 1/4 + 1/8
    # enumeration: every accept/reject pattern of gamma independent drafts, weighted by its
    # probability, emits (length of the leading run of accepts) + 1 tokens
    for gamma in (1, 2, 3, 5):
        for a in (0.3, 0.8):
            tot = 0.0
            for pat in itertools.product([0, 1], repeat=gamma):
                pr = 1.0
                for b in pat:
                    pr *= a if b else (1 - a)
                run = 0
                while run < gamma and pat[run]:
                    run += 1
                tot += pr * (run + 1)
            assert abs(tot - O.expected_tokens_per_round(a, gamma)) < 1e-12


def test_speed_model_hand_worked():
    # all drafts accepted: gamma + 1 tokens in gamma * t_draft + t_verify (the paper's example)
    n, rate, sp = O.speed_model(1.0, 4, 1.0, 2.0, 2.0)
    assert (n, rate) == (5.0, 5.0 / 6.0) and abs(sp - 10.0 / 6.0) < 1e-15
    # nothing accepted: one token per round, slower than plain decoding by the drafting time
    n, rate, sp = O.speed_model(0.0, 4, 1.0, 2.0, 2.0)
    assert (n, rate) == (1.0, 1.0 / 6.0) and abs(sp - 2.0 / 6.0) < 1e-15
    # no drafting at all is plain decoding when the verification of one column costs t_plain
    assert O.speed_model(0.7, 0, 1.0, 2.0, 2.0) == (1.0, 0.5, 1.0)
    # swapping the two times must change the answer (gamma multiplies the draft time only)
    assert abs(O.speed_model(0.5, 3, 1.0, 4.0, 1.0)[1] - 1.875 / 7.0) < 1e-15
    assert abs(O.speed_model(0.5, 3, 4.0, 1.0, 1.0)[1] - 1.875 / 13.0) < 1e-15


def test_tune_measured_hand_worked():
    # equal acceptance: the fastest format wins; equal times: the best accepted one wins
    al = [[0.8, 0.8], [0.8, 0.8]]
    td = [[2.0, 1.5], [1.0, 1.2]]
    tv = [[3.0, 3.0], [3.0, 3.0]]
    assert O.tune_measured(al, td, tv, 4) == (1, 0)
    assert O.tune_measured([[0.5, 0.9], [0.7, 0.6]], [[1.0, 1.0], [1.0, 1.0]], tv, 4) == (0, 1)
    # a trade worked by hand, gamma = 2: (alpha .9, t_d 2, t_v 4): (1 + .9 + .81) / 8 = 0.33875;
    # (alpha .6, t_d 1, t_v 4): (1 + .6 + .36) / 6 = 0.32667 -> the first; with t_d = 0.9 for the second:
    # 1.96 / 5.8 = 0.33793 -> still the first; with t_d = 0.8: 1.96 / 5.6 = 0.35 -> the second
    assert O.tune_measured([[0.9, 0.6]], [[2.0, 1.0]], [[4.0, 4.0]], 2) == (0, 0)
    assert O.tune_measured([[0.9, 0.6]], [[2.0, 0.9]], [[4.0, 4.0]], 2) == (0, 0)
    assert O.tune_measured([[0.9, 0.6]], [[2.0, 0.8]], [[4.0, 4.0]], 2) == (0, 1)
    # equals: first in row-major order
    assert O.tune_measured([[0.5, 0.5], [0.5, 0.5]], [[1.0, 1.0], [1.0, 1.0]], [[1.0, 1.0], [1.0, 1.0]], 3) == (0, 0)


def test_token_prob_closed_forms():
    # uniform logits: 1 / V; two logits: the logistic function; shift invariance; sums to one
    assert abs(O.token_prob(np.zeros(10), 3) - 0.1) < 1e-15
    assert abs(O.token_prob(np.full(7, 123.0), 0) - 1.0 / 7.0) < 1e-15
    for d in (-3.0, 0.0, 0.5, 20.0):
        assert abs(O.token_prob([0.0, d], 1) - 1.0 / (1.0 + math.exp(-d))) < 1e-15
    z = np.array([0.3, -1.2, 2.5, 0.0, 700.0])           # exp(700) overflows unless the maximum is subtracted
    assert abs(O.token_prob(z, 4) - 1.0) < 1e-12 and O.token_prob(z, 0) < 1e-300
    z = np.array([0.3, -1.2, 2.5, 0.0])
    assert abs(sum(O.token_prob(z, i) for i in range(4)) - 1.0) < 1e-15
    assert abs(O.token_prob(z + 11.0, 2) - O.token_prob(z, 2)) < 1e-15
    # hand-worked: logits ln 1, ln 2, ln 5 -> 1/8, 2/8, 5/8
    z = np.log(np.array([1.0, 2.0, 5.0]))
    assert [round(O.token_prob(z, i), 12) for i in range(3)] == [0.125, 0.25, 0.625]
    # against the library routine
    import torch
    z = np.random.Generator(np.random.Philox(3)).standard_normal(1000) * 4
    ref = torch.softmax(torch.from_numpy(z), dim=0).numpy()
    assert max(abs(O.token_prob(z, i) - ref[i]) for i in (0, 17, 999)) < 1e-15


def test_sampling_round_against_its_parts():
    """The sampling round is the draft passes, the verification pass, token_prob and Eq. 1 put
    together: with r = 0 everything is accepted (0 > p/q never holds), with r just below 1 a draft
    is rejected exactly where the target gives it less probability than the draft model, and the
    emitted tokens are the greedy round's whenever n agrees."""
    import synth
    shape = synth.TINY
    weights = synth.model_weights(shape, seed=1)
    tab = synth.rope_table(64, shape.head_dim, shape.rope_theta)
    prompt = synth.token_ids(5, shape.vocab, seed=5)
    k = 3

    def fresh():
        om = O.OracleModel(shape, weights, tab, w_keep=600, w_t=4, kv_keep=600, kv_t=4)
        return om, O.prefill(om, prompt)

    om, pending = fresh()
    n, emitted, p, q = O.spec_round_sampling(om, pending, k, [0.0] * k)
    assert n == k and len(emitted) == k + 1 and om.cache_len() == len(prompt) - 1 + k + 1
    assert all(0.0 < x <= 1.0 for x in p + q)
    om2, pending2 = fresh()
    r = [1.0 - 1e-12] * k
    n2, emitted2, p2, q2 = O.spec_round_sampling(om2, pending2, k, r)
    assert p2 == p and q2 == q
    want = next((i for i in range(k) if p[i] < q[i] * r[i]), k)
    assert n2 == want and emitted2[:n2] == emitted[:n2] and om2.cache_len() == len(prompt) - 1 + n2 + 1
