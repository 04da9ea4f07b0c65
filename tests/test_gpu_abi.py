"""Behaviour of the C ABI as the header states it: requests outside the limits come back as an
error code from the host-side checks, before any kernel is launched; and the library used from
a plain C program."""
import copy
import ctypes as C

import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_26558_amd import binding as B
    return torch, B, B.Context()


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def _code(B, fn):
    with pytest.raises(B.CasError) as e:
        fn()
    return e.value.code


def test_linear_entry_points_reject_what_they_cannot_do(env):
    torch, B, ctx = env
    lib = B._lib()
    ew = B.cas_encode_weight(ctx, _dev(torch, synth.weight_matrix(32, 256, seed=1)), 600, 4)
    X = _dev(torch, synth.activations(256, 33, seed=2))
    y = torch.empty((33, 32), device="cuda")
    # batch and column limits
    assert lib.cas_gemv_draft(ctx.h, C.byref(ew.desc), B._ptr(ew.spec), B._ptr(X), 5, B._ptr(y)) == B.CAS_EINVAL
    assert lib.cas_gemv_draft(ctx.h, C.byref(ew.desc), B._ptr(ew.spec), B._ptr(X), 0, B._ptr(y)) == B.CAS_EINVAL
    assert lib.cas_gemm_verify(ctx.h, C.byref(ew.desc), B._ptr(ew.spec), B._ptr(ew.verif), B._ptr(X), 33,
                               B._ptr(y)) == B.CAS_EINVAL
    # a speculation buffer that is not 256-byte aligned, a missing buffer
    off = C.c_void_p(ew.spec.data_ptr() + 64)
    assert lib.cas_gemv_draft(ctx.h, C.byref(ew.desc), off, B._ptr(X), 1, B._ptr(y)) == B.CAS_EINVAL
    assert lib.cas_gemm_verify(ctx.h, C.byref(ew.desc), B._ptr(ew.spec), None, B._ptr(X), 1, B._ptr(y)) == B.CAS_EINVAL
    # a descriptor whose stream widths do not belong to its shape
    bad = copy.copy(ew.desc)
    bad.sw += 1
    assert lib.cas_gemv_draft(ctx.h, C.byref(bad), B._ptr(ew.spec), B._ptr(X), 1, B._ptr(y)) == B.CAS_EINVAL
    # the valid call still works afterwards
    assert B.cas_gemv_draft(ctx, ew, X[:1].contiguous()).shape == (1, 32)


def test_rows_too_long_for_the_lds_are_not_supported(env):
    torch, B, ctx = env
    cols = 49152           # 48 K fp32 activations + segment padding exceed one workgroup's LDS
    W = torch.zeros((2, cols), dtype=torch.int16, device="cuda")
    ew = B.cas_encode_weight(ctx, W, 600, 4)
    x = torch.zeros((1, cols), dtype=torch.int16, device="cuda")
    assert _code(B, lambda: B.cas_gemv_draft(ctx, ew, x)) == B.CAS_ENOTSUP
    mw = B.cas_mx_encode(ctx, ew)
    assert _code(B, lambda: B.cas_gemv_draft_mx(ctx, mw, x)) == B.CAS_ENOTSUP


def test_shared_exponent_descriptor_is_checked(env):
    torch, B, ctx = env
    lib = B._lib()
    ew = B.cas_encode_weight(ctx, _dev(torch, synth.weight_matrix(8, 96, seed=3)), 600, 4)
    mw = B.cas_mx_encode(ctx, ew)
    x = _dev(torch, synth.activations(96, 1, seed=4))
    y = torch.empty(8, device="cuda")
    bad = copy.copy(mw.desc)
    bad.off_field += 256
    assert lib.cas_gemv_draft_mx(ctx.h, C.byref(bad), B._ptr(mw.spec), B._ptr(x), B._ptr(y)) == B.CAS_EINVAL
    assert lib.cas_mx_decode(ctx.h, C.byref(mw.desc), B._ptr(mw.spec), None, B._ptr(y), 95) == B.CAS_EINVAL  # ld < cols
    with pytest.raises(B.CasError):
        d = copy.copy(ew.desc); d.t = 9
        B.cas_mx_plan(d)


def test_attention_limits(env):
    torch, B, ctx = env
    kv = B.KVCache(ctx, 1, 2, n_pages=2, max_seqs=1, max_pages_per_seq=2)
    z = lambda *s: torch.zeros(s, dtype=torch.int16, device="cuda")
    # 17 columns; a head count that is no multiple of the kv heads; fewer in-flight vectors than columns
    assert _code(B, lambda: B.cas_attention(ctx, kv, 0, 0, True, z(17, 2, 128), z(17, 2, 128), z(17, 2, 128))) == B.CAS_EINVAL
    assert _code(B, lambda: B.cas_attention(ctx, kv, 0, 0, True, z(1, 3, 128), z(1, 2, 128), z(1, 2, 128))) == B.CAS_EINVAL
    assert _code(B, lambda: B.cas_attention(ctx, kv, 0, 0, False, z(2, 2, 128), z(1, 2, 128), z(1, 2, 128))) == B.CAS_EINVAL
    # layer and sequence out of range
    assert _code(B, lambda: B.cas_attention(ctx, kv, 1, 0, False, z(1, 2, 128), z(1, 2, 128), z(1, 2, 128))) == B.CAS_EINVAL
    assert _code(B, lambda: B.cas_attention(ctx, kv, 0, 1, False, z(1, 2, 128), z(1, 2, 128), z(1, 2, 128))) == B.CAS_EINVAL
    # appending past the pages a sequence may hold
    assert _code(B, lambda: B.cas_kv_append(ctx, kv, 0, 0, z(129, 2, 128), z(129, 2, 128))) == B.CAS_ENOMEM


def test_entry_points_added_later_reject_what_they_cannot_do(env):
    """cas_attention_multi, cas_token_probs, cas_spec_round_sampling and cas_dense_decode_step:
    argument errors come back as codes from the host-side checks; degenerate sizes work."""
    torch, B, _ = env
    lib = B._lib()
    ctx = B.Context(workspace=torch.empty(8 << 20, dtype=torch.uint8, device="cuda"))
    kv = B.KVCache(ctx, 1, 2, n_pages=4, max_seqs=2, max_pages_per_seq=2)
    z = lambda *s: torch.zeros(s, dtype=torch.int16, device="cuda")
    # the same sequence twice in one call; a sequence out of range
    q, kn = [z(1, 2, 128), z(1, 2, 128)], [z(1, 2, 128), z(1, 2, 128)]
    assert _code(B, lambda: B.cas_attention_multi(ctx, kv, 0, [0, 0], False, q, kn, kn)) == B.CAS_EINVAL
    assert _code(B, lambda: B.cas_attention_multi(ctx, kv, 0, [0, 2], False, q, kn, kn)) == B.CAS_EINVAL
    outs = B.cas_attention_multi(ctx, kv, 0, [0, 1], False, q, kn, kn)       # empty caches, one in-flight vector each
    assert len(outs) == 2 and outs[0].shape == (1, 2, 128)
    # probabilities: no rows is fine, a vocabulary of 0 is not
    lg = torch.zeros((0, 8), dtype=torch.float32, device="cuda")
    assert B.cas_token_probs(ctx, lg, torch.zeros(0, dtype=torch.int32, device="cuda")).numel() == 0
    one = torch.zeros((1, 1), dtype=torch.float32, device="cuda")
    assert float(B.cas_token_probs(ctx, one, torch.zeros(1, dtype=torch.int32, device="cuda"))[0]) == 1.0
    assert lib.cas_token_probs(ctx.h, B._ptr(one), 0, 1, B._ptr(one), B._ptr(one)) == B.CAS_EINVAL
    assert lib.cas_spec_round_sampling_scratch_floats(100, 3) == 7 * 100 + 6
    assert lib.cas_spec_round_sampling_scratch_floats(0, 3) == 0
    # the rounds and the plain bf16 step on a small model
    shape = synth.TINY
    weights = synth.model_weights(shape, seed=1)
    dev = lambda a: _dev(torch, a)
    layers = []
    for lw in weights["layers"]:
        L = {n: B.cas_encode_weight(ctx, dev(lw[n]), 600, 4) for n in ("wqkv", "wo", "wgu", "wd")}
        L["g_attn"], L["g_ffn"] = dev(lw["g_attn"]), dev(lw["g_ffn"])
        layers.append(L)
    head = B.cas_encode_weight(ctx, dev(weights["lm_head"]), 600, 4)
    rope = torch.from_numpy(synth.rope_table(64, shape.head_dim, shape.rope_theta)).cuda()
    model = B.Model(ctx, shape, layers, head, dev(weights["embed"]), dev(weights["g_final"]), rope, 4)
    kv = B.KVCache(ctx, shape.n_layers, shape.n_kv_heads, n_pages=1, max_seqs=1, max_pages_per_seq=1)
    # a draft length that does not fit max_cols; k = 0 is a plain step that needs no scratch and no r
    assert _code(B, lambda: B.cas_spec_round_sampling(ctx, model, kv, 0, 1, 4, [0.5] * 4)) == B.CAS_EINVAL
    n, out, p, q = B.cas_spec_round_sampling(ctx, model, kv, 0, 1, 0, [])
    assert n == 0 and len(out) == 1 and B.cas_kv_len(kv, 0) == 1
    dense = [{n: dev(lw[n]) for n in ("wqkv", "wo", "wgu", "wd")} for lw in weights["layers"]]
    kvd = shape.n_kv_heads * shape.head_dim
    kc = torch.zeros((shape.n_layers, 64, kvd), dtype=torch.int16, device="cuda")
    tin = torch.ones(1, dtype=torch.int32, device="cuda")
    # a position past the model's table; a missing matrix
    assert _code(B, lambda: B.cas_dense_decode_step(ctx, model, dense, dev(weights["lm_head"]), kc, kc.clone(), 64, tin)) == B.CAS_EINVAL
    arr = (B.cas_dense_layer * shape.n_layers)()
    assert lib.cas_dense_decode_step(ctx.h, model.h, arr, B._ptr(kc), B._ptr(kc), B._ptr(kc), 0, B._ptr(tin), None,
                                     None) == B.CAS_EINVAL
    # without a workspace for the attention partials the step says so
    ctx0 = B.Context()
    model0 = B.Model(ctx0, shape, layers, head, dev(weights["embed"]), dev(weights["g_final"]), rope, 4)
    assert _code(B, lambda: B.cas_dense_decode_step(ctx0, model0, dense, dev(weights["lm_head"]), kc, kc.clone(), 0, tin)) == B.CAS_ENOMEM


def test_exponent_form_entry_points_reject_what_they_cannot_do(env):
    """cas_gemm_verify_unary, cas_gemm_verify_mx, cas_model_use_unary / _mx and the shared-exponent
    cache: argument errors come back as codes from the host-side checks; degenerate sizes work."""
    torch, B, _ = env
    lib = B._lib()
    ctx = B.Context(workspace=torch.empty(4 << 20, dtype=torch.uint8, device="cuda"))
    dev = lambda a: _dev(torch, a)
    W = synth.weight_matrix(32, 256, seed=3)
    ew = B.cas_encode_weight(ctx, dev(W), 600, 4)
    uw, mw = B.cas_unary_encode(ctx, ew), B.cas_mx_encode(ctx, ew)
    X = dev(synth.activations(256, 2, seed=4))
    Y = torch.empty((2, 32), dtype=torch.float32, device="cuda")

    for fn, d, spec, verif in ((lib.cas_gemm_verify_unary, uw.desc, uw.uspec, uw.verif),
                               (lib.cas_gemm_verify_mx, mw.desc, mw.spec, mw.verif)):
        args = lambda **k: (ctx.h, C.byref(d), k.get("spec", B._ptr(spec)), k.get("verif", B._ptr(verif)),
                            k.get("X", B._ptr(X)), k.get("ncols", 2), k.get("Y", B._ptr(Y)))
        assert fn(*args()) == B.CAS_OK
        assert fn(*args(ncols=0)) == B.CAS_EINVAL and fn(*args(ncols=33)) == B.CAS_EINVAL
        assert fn(*args(spec=None)) == B.CAS_EINVAL and fn(*args(verif=None)) == B.CAS_EINVAL
        assert fn(*args(X=None)) == B.CAS_EINVAL and fn(*args(Y=None)) == B.CAS_EINVAL
        assert fn(*args(spec=spec.data_ptr() + 4)) == B.CAS_EINVAL          # not 256-byte aligned
        assert fn(None, *args()[1:]) == B.CAS_EINVAL
    # without a workspace the unary form has nowhere to put its re-coded rows; the shared-exponent form needs none
    ctx0 = B.Context()
    assert _code(B, lambda: B.cas_gemm_verify_unary(ctx0, uw, X)) == B.CAS_ENOMEM
    np.testing.assert_array_equal(B.cas_gemm_verify_mx(ctx0, mw, X).cpu().numpy(),
                                  B.cas_gemm_verify_mx(ctx, mw, X).cpu().numpy())
    # an empty matrix
    e = B.cas_encode_weight(ctx, torch.empty((0, 256), dtype=torch.int16, device="cuda"), 600, 4)
    assert B.cas_gemm_verify_mx(ctx, B.cas_mx_encode(ctx, e), X).shape == (2, 0)
    assert B.cas_gemm_verify_unary(ctx, B.cas_unary_encode(ctx, e), X).shape == (2, 0)
    # the model: a layer or tensor that does not exist, a form of another matrix, a NULL buffer
    shape = synth.TINY
    weights = synth.model_weights(shape, seed=1)
    layers = []
    for lw in weights["layers"]:
        L = {n: B.cas_encode_weight(ctx, dev(lw[n]), 600, 4) for n in ("wqkv", "wo", "wgu", "wd")}
        L["g_attn"], L["g_ffn"] = dev(lw["g_attn"]), dev(lw["g_ffn"])
        layers.append(L)
    head = B.cas_encode_weight(ctx, dev(weights["lm_head"]), 600, 4)
    rope = torch.from_numpy(synth.rope_table(64, shape.head_dim, shape.rope_theta)).cuda()
    model = B.Model(ctx, shape, layers, head, dev(weights["embed"]), dev(weights["g_final"]), rope, 4)
    uq, mq = B.cas_unary_encode(ctx, layers[0]["wqkv"]), B.cas_mx_encode(ctx, layers[0]["wqkv"])
    assert _code(B, lambda: model.use_unary(shape.n_layers, 0, uq)) == B.CAS_EINVAL
    assert _code(B, lambda: model.use_unary(0, 4, uq)) == B.CAS_EINVAL
    assert _code(B, lambda: model.use_unary(0, 1, uq)) == B.CAS_EINVAL       # wqkv's form offered for wo
    assert _code(B, lambda: model.use_mx(0, 3, mq)) == B.CAS_EINVAL          # ... and for wd
    assert lib.cas_model_use_unary(model.h, 0, 0, C.byref(uq.desc), None) == B.CAS_EINVAL
    assert lib.cas_model_use_mx(model.h, 0, 0, C.byref(mq.desc), B._ptr(mq.spec), None) == B.CAS_EINVAL
    assert lib.cas_model_use_unary(None, 0, 0, None, None) == B.CAS_EINVAL
    model.use_unary(0, 0, uq); model.use_mx(0, 0, mq); model.use_mx(0, 0, None)   # the last call wins; switching off works
    # the cache: a mode without kernels
    d = B.cas_kv_desc()
    d.n_layers, d.n_kv_heads, d.head_dim, d.page_tokens, d.n_pages, d.max_seqs, d.max_pages_per_seq = 1, 1, 128, 64, 1, 1, 1
    d.fmt = B.cas_fmt(600, 4, 1)
    assert lib.cas_kv_desc_init(C.byref(d)) == B.CAS_ENOTSUP


def test_library_from_a_plain_c_program():
    """tests/c/abi_gpu_roundtrip.c: encode, exact and draft reconstruction, draft GEMV and
    verification GEMM through the C ABI with device memory from the HIP runtime, no Python in the
    path.  The program is built with the library (built here if it is missing)."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "tests", "c", "abi_gpu_roundtrip")
    if not os.path.exists(exe):
        import __graft_entry__ as g
        exe = g.build_c_program()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi gpu roundtrip ok" in r.stdout
