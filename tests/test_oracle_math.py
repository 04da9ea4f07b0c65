"""Pins of the oracle's arithmetic: GEMV/GEMM, attention, decoder ops, acceptance,
speculative vs plain token streams.  CPU only."""
import itertools

import numpy as np
import pytest
import torch

from oracle import cassandra_oracle as O
import synth


def _t64(u16):
    return torch.tensor(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).to(torch.float64)


def test_gemv_identity_config_equals_plain_bf16_gemv():
    """keep everything, truncate nothing: the draft is the target (Sec. 4.1)."""
    w = synth.weight_matrix(48, 160, seed=1)
    x = synth.activations(160, 1, seed=2)[0]
    p = O.encode_weight(w, 1000, 0)
    ref = (_t64(w) @ _t64(x)).numpy()
    np.testing.assert_array_equal(O.gemv_draft(p, x), ref)
    np.testing.assert_array_equal(O.gemm_verify(p, x[None])[0], ref)


@pytest.mark.parametrize("keep,t", [(600, 4), (250, 4), (500, 0), (1000, 5)])
def test_gemm_verify_is_gemm_of_the_original_weights(keep, t):
    w = synth.weight_matrix(64, 300, seed=3)
    X = synth.activations(300, 5, seed=4)
    a = synth.act_norm(300, seed=5)
    p = O.encode_weight(w, keep, t, a)
    ref = (_t64(X) @ _t64(w).T).numpy()
    got = O.gemm_verify(p, X)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    # each column equals the one-column call bit for bit (Sec. 2.2: batched verification)
    for c in range(5):
        np.testing.assert_array_equal(got[c], O.gemm_verify(p, X[c:c + 1])[0])


def test_gemv_draft_probes_columns_of_the_draft_weights():
    """x = unit vector j reads column j: kept entries are the truncated weights, the rest 0."""
    w = synth.weight_matrix(32, 96, seed=6)
    p = O.encode_weight(w, 600, 4)
    mask = O.unpack_mask(p)
    one = np.uint16(0x3F80)
    for j in (0, 17, 95):
        x = np.zeros(96, dtype=np.uint16)
        x[j] = one
        y = O.gemv_draft(p, x)
        expect = np.where(mask[:, j], _t64(w[:, j] & np.uint16(0xFFF0)).numpy(), 0.0)
        np.testing.assert_array_equal(y, expect)
    # draft error is bounded by the dropped part: |W - Wd| <= |W| 2^-3 at kept, |W| at pruned
    wd = O.bf16_to_f64(O.decode_draft(p)); wf = O.bf16_to_f64(w)
    assert (np.abs(wf - wd)[mask] <= np.abs(wf)[mask] * 2.0 ** -3).all()


def test_attention_special_cases_and_library():
    rng = np.random.default_rng(0)
    d, nq, nkv, T = 128, 4, 2, 37
    q = synth.normal_bf16((nq, d), 1.0, seed=7)
    k = synth.kv_tensor(T, nkv, d, seed=8)
    v = synth.kv_tensor(T, nkv, d, seed=9, outlier_channels=0)
    # context length 1: the output is v itself
    o = O.attention(q, k[:1], v[:1], nq, nkv)
    for h in range(nq):
        np.testing.assert_array_equal(o[h], v[0, h // 2])
    # equal scores (q = 0): mean of V
    o = O.attention(np.zeros_like(q), k, v, nq, nkv)
    for h in range(nq):
        np.testing.assert_array_equal(o[h], O.f64_to_bf16(O.bf16_to_f64(v[:, h // 2]).mean(axis=0)))
    # general: library scaled-dot-product attention in float64
    o = O.attention(q, k, v, nq, nkv)
    kq = _t64(k).permute(1, 0, 2).repeat_interleave(2, dim=0)
    vq = _t64(v).permute(1, 0, 2).repeat_interleave(2, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(_t64(q)[:, None, :], kq, vq)[:, 0, :]
    np.testing.assert_allclose(O.bf16_to_f64(o), ref.numpy(), rtol=2.0 ** -8, atol=1e-30)


def test_decoder_ops_against_library():
    h = synth.normal_bf16((256,), 2.0, seed=10)
    g = synth.normal_bf16((256,), 1.0, seed=11)
    ref = torch.nn.functional.rms_norm(_t64(h), (256,), _t64(g), eps=1e-5)
    got = O.bf16_to_f64(O.rmsnorm(h, g, 1e-5))
    np.testing.assert_allclose(got, ref.numpy(), rtol=2.0 ** -8)
    gate = np.linspace(-6, 6, 97); up = np.linspace(2, -3, 97)
    gb, ub = O.round_bf16(gate), O.round_bf16(up)
    ref = (torch.nn.functional.silu(torch.tensor(gb)) * torch.tensor(ub)).numpy()
    np.testing.assert_allclose(O.bf16_to_f64(O.swiglu(gate, up)), ref, rtol=2.0 ** -8, atol=1e-30)
    # residual add: against the library's bf16 tensors, addend rounded, then the sum (the
    # hand-worked cases that separate other readings are in test_oracle_pins.py)
    y = np.array([0.1, -3.7, 1e-3])
    hh = O.f64_to_bf16(np.array([1.0, 2.0, -4.0]))
    ref = (torch.tensor([1.0, 2.0, -4.0], dtype=torch.bfloat16) + torch.tensor(y).to(torch.bfloat16))
    np.testing.assert_array_equal(O.add_bf16(hh, y).view(np.int16), ref.view(torch.int16).numpy())


def test_rope_is_a_rotation_by_position_angle():
    tab = synth.rope_table(64, 128, 500000.0)
    x = synth.normal_bf16((3, 128), 1.0, seed=12)
    np.testing.assert_array_equal(O.rope(x, 0, tab), x)                 # angle 0
    xf = O.bf16_to_f64(x)
    z = xf[:, :64] + 1j * xf[:, 64:]
    pos = 29
    inv = 500000.0 ** (-np.arange(64) * 2.0 / 128)
    zr = z * np.exp(1j * pos * inv)[None, :]
    got = O.bf16_to_f64(O.rope(x, pos, tab))
    np.testing.assert_allclose(got[:, :64], zr.real, rtol=0, atol=2.0 ** -7 * np.abs(zr).max())
    np.testing.assert_allclose(got[:, 64:], zr.imag, rtol=0, atol=2.0 ** -7 * np.abs(zr).max())


def test_accept_brute_force_against_definition():
    """n = number of leading positions where draft and target agree; emit those drafts and
    the target's next token (Sec. 2.2 greedy rule)."""
    for k in range(0, 5):
        for d in itertools.product(range(3), repeat=k):
            for t in itertools.product(range(3), repeat=k + 1):
                n, out = O.accept_greedy(list(d), list(t))
                n_def = max(m for m in range(k + 1) if all(d[i] == t[i] for i in range(m)))
                assert n == n_def
                assert out == list(t[: n + 1])        # accepted drafts equal the target's tokens
                assert len(out) == n + 1


def _tiny_model(keep, t, seed=1):
    shape = synth.TINY
    w = synth.model_weights(shape, seed)
    tab = synth.rope_table(128, shape.head_dim, shape.rope_theta)
    return O.OracleModel(shape, w, tab, w_keep=keep, w_t=t, kv_keep=keep, kv_t=t)


@pytest.mark.parametrize("keep,t,k", [(600, 4, 4), (250, 4, 3), (1000, 0, 4), (800, 2, 1)])
def test_speculative_stream_equals_plain_stream(keep, t, k):
    """Greedy speculative decoding preserves the target model's output exactly (Sec. 2.2)."""
    prompt = synth.token_ids(6, synth.TINY.vocab, seed=5)
    n_new = 10
    plain = O.plain_decode(_tiny_model(keep, t), prompt, n_new)
    stats = []
    spec = O.spec_decode(_tiny_model(keep, t), prompt, n_new, k, stats)
    assert spec == plain
    if keep == 1000 and t == 0:
        assert all(n == k for n in stats)             # draft model == target model
    assert all(0 <= n <= k for n in stats)


def test_cache_is_lossless_and_draft_cache_is_the_prefix():
    m = _tiny_model(600, 4)
    prompt = synth.token_ids(5, synth.TINY.vocab, seed=6)
    _, kv = m.forward(prompt, draft=False)
    m.append_kv(kv, 5)
    ck, cv = m._cache_kv(0, draft=False)
    np.testing.assert_array_equal(ck, kv[0][0])
    np.testing.assert_array_equal(cv, kv[0][1])
    dk, _ = m._cache_kv(0, draft=True)
    assert (((dk ^ ck) < 16) | (dk == 0)).all()
    assert ((dk != 0).sum(axis=-1) <= 77).all()


def test_accept_sampling_against_definition_brute_force():
    """Eq. 1 on every combination of a small grid of ratios and random numbers: the result is the
    index of the first rejected draft, or gamma; p = q accepts everything; p = 0 rejects at once."""
    grid_ratio = [0.0, 0.3, 1.0, 2.5]
    grid_r = [0.0, 0.29, 0.31, 0.99]
    for gamma in range(0, 4):
        for ratios in itertools.product(grid_ratio, repeat=gamma):
            for rs in itertools.product(grid_r, repeat=gamma):
                q = [0.4] * gamma
                p = [x * 0.4 for x in ratios]
                n = O.accept_sampling(p, q, rs)
                first_rej = next((i for i in range(gamma) if rs[i] > ratios[i]), gamma)
                assert n == first_rej
    assert O.accept_sampling([0.2, 0.5], [0.2, 0.5], [0.999, 0.999]) == 2
    assert O.accept_sampling([0.0, 0.5], [0.2, 0.5], [0.001, 0.0]) == 0
