"""GPU parity of the shared-exponent (MX) form of the speculation data (Sec. 4.2 exponent
compression, first approach; Sec. 5.1 decoder #N) against the oracle, through the C ABI: every
region of both buffers bit for bit, both reconstructions, the draft GEMV and the verification
GEMM on the converted matrix."""
import numpy as np
import pytest

from oracle import cassandra_oracle as O
import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_26558_amd import binding as B
    return torch, B, B.Context(workspace=torch.empty(8 << 20, dtype=torch.uint8, device="cuda"))


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def _regions(mw):
    m, d = mw.desc, mw.desc.base
    s, v = mw.spec.cpu().numpy(), mw.verif.cpu().numpy()
    def words(b, off, n, w):
        return b[off: off + 4 * n * w].view("<u4").reshape(n, w)
    sexp = s[m.off_sexp: m.off_sexp + d.rows * m.ew].reshape(d.rows, m.ew)
    return (words(s, m.off_bitmap, d.rows, d.bw), sexp, words(s, m.off_field, d.rows, m.fw),
            words(v, m.off_lo, d.rows, d.lw), words(v, m.off_pruned, d.rows, d.pw))


CASES = [
    # rows, cols, keep, t, arbitrary bit patterns mixed in
    (37, 77, 600, 4, False),
    (16, 128, 600, 4, True),
    (5, 1, 1000, 4, False),
    (70, 4096, 600, 4, False),
    (33, 2500, 250, 0, True),
    (20, 300, 0, 4, False),
    (20, 300, 1000, 7, True),
    (9, 14336, 600, 3, False),
    (300, 64, 500, 5, True),
    (1400, 512, 600, 4, False),     # more workgroups than CUs
]


def _matrix(rows, cols, special, seed):
    """Weights whose magnitudes spread over several binades inside a block; `special` adds
    arbitrary 16-bit patterns (rare exponents, subnormals, zeros, Inf, NaN)."""
    rng = np.random.Generator(np.random.Philox(seed + 1))
    W = synth.weight_matrix(rows, cols, seed=seed)
    scale = np.exp2(rng.integers(-6, 1, size=W.shape).astype(np.float64))
    W = O.f64_to_bf16(O.bf16_to_f64(W) * scale)
    if special:
        idx = rng.integers(0, W.size, size=min(W.size, 96))
        W.reshape(-1)[idx] = rng.integers(0, 65536, size=idx.shape).astype(np.uint16)
        W.reshape(-1)[idx[:5]] = np.array([0x7F80, 0xFFFF, 0x0001, 0x8000, 0x0080], dtype=np.uint16)[: len(idx[:5])]
    return W


@pytest.mark.parametrize("rows,cols,keep,t,special", CASES)
def test_mx_buffers_and_reconstruction_bit_exact(env, rows, cols, keep, t, special):
    torch, B, ctx = env
    print(f"case rows={rows} cols={cols} keep={keep} t={t} special={special}", flush=True)
    W = _matrix(rows, cols, special, seed=rows + cols + t)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), keep, t)
    mw = B.cas_mx_encode(ctx, ew)
    torch.cuda.synchronize()
    p = O.encode_weight(W, keep, t)
    m = O.to_mx(p)
    assert mw.desc.fw == m.field.shape[1] and mw.desc.base.lw == m.lo.shape[1]
    bm, sexp, field, lo, pruned = _regions(mw)
    np.testing.assert_array_equal(bm, p.bitmap)
    np.testing.assert_array_equal(sexp[:, : p.bitmap.shape[1]], m.sexp)
    assert (sexp[:, p.bitmap.shape[1]:] == 0).all()
    np.testing.assert_array_equal(field, m.field)
    np.testing.assert_array_equal(lo, m.lo)
    np.testing.assert_array_equal(pruned, p.pruned)
    full = B.cas_mx_decode(ctx, mw, full=True).cpu().numpy().view(np.uint16)
    draft = B.cas_mx_decode(ctx, mw, full=False).cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(full, O.decode_full_mx(m))
    np.testing.assert_array_equal(draft, O.decode_draft_mx(m))


@pytest.mark.parametrize("rows,cols,keep,t,special", [c for c in CASES if not c[4]])
def test_gemv_draft_mx_matches_oracle(env, rows, cols, keep, t, special):
    torch, B, ctx = env
    print(f"case rows={rows} cols={cols} keep={keep} t={t}", flush=True)
    W = _matrix(rows, cols, False, seed=rows + cols + t)
    x = synth.activations(cols, 1, seed=11)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), keep, t)
    mw = B.cas_mx_encode(ctx, ew)
    y = B.cas_gemv_draft_mx(ctx, mw, _dev(torch, x)).cpu().numpy()
    ref = O.gemv_draft_mx(O.to_mx(O.encode_weight(W, keep, t)), x[0])
    tol = np.linalg.norm(O.bf16_to_f64(W), axis=1) * np.linalg.norm(O.bf16_to_f64(x[0])) + 1e-30
    err = np.abs(y - ref) / tol
    assert err.max() < 2e-3          # spec bar
    assert err.max() < 2e-5, err.max()


def test_gemv_draft_mx_tiny_magnitudes(env):
    """Blocks whose shared exponent is near the bottom of the range: the per-block scale is a
    subnormal float and must not be flushed."""
    torch, B, ctx = env
    rng = np.random.Generator(np.random.Philox(5))
    W = ((rng.integers(0, 2, (24, 256)) << 15) | (rng.integers(0, 5, (24, 256)) << 7)
         | rng.integers(0, 128, (24, 256))).astype(np.uint16)
    x = synth.activations(256, 1, seed=3)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), 600, 4)
    mw = B.cas_mx_encode(ctx, ew)
    y = B.cas_gemv_draft_mx(ctx, mw, _dev(torch, x)).cpu().numpy().astype(np.float64)
    ref = O.gemv_draft_mx(O.to_mx(O.encode_weight(W, 600, 4)), x[0])
    assert np.abs(ref).max() > 0
    tol = np.linalg.norm(O.bf16_to_f64(W), axis=1) * np.linalg.norm(O.bf16_to_f64(x[0]))
    assert (np.abs(y - ref) <= 2e-5 * tol + 2.0 ** -149).all()


@pytest.mark.parametrize("ncols", [1, 5, 20])
@pytest.mark.parametrize("rows,cols,keep,t,special", [c for c in CASES if not c[4]])
def test_gemm_verify_mx_is_the_product_with_the_converted_matrix(env, rows, cols, keep, t, special, ncols):
    """Verification on the shared-exponent form (Sec. 4.2 MX approach under Sec. 4.1 target
    inference): Y = W' X with W' the oracle's converted matrix."""
    torch, B, ctx = env
    print(f"case rows={rows} cols={cols} keep={keep} t={t} ncols={ncols}", flush=True)
    W = _matrix(rows, cols, False, seed=rows + cols + t)
    X = synth.activations(cols, ncols, seed=13)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), keep, t)
    mw = B.cas_mx_encode(ctx, ew)
    Y = B.cas_gemm_verify_mx(ctx, mw, _dev(torch, X)).cpu().numpy()
    Wc = O.decode_full_mx(O.to_mx(O.encode_weight(W, keep, t)))
    Wf = O.bf16_to_f64(Wc)
    ref = (Wf @ O.bf16_to_f64(X).T).T
    tol = np.linalg.norm(Wf, axis=1)[None, :] * np.linalg.norm(O.bf16_to_f64(X), axis=1)[:, None] + 1e-30
    err = np.abs(Y - ref) / tol
    assert err.max() < 2e-3          # spec bar
    assert err.max() < 2e-5, err.max()
    # a unit vector picks one column of the converted matrix: exact, every bit of the re-coding counts
    if ncols == 5:
        picks = sorted({0, cols - 1, cols // 2, min(33, cols - 1), min(31, cols - 1)})[:5]
        U = np.zeros((len(picks), cols), dtype=np.uint16)
        for i, j in enumerate(picks):
            U[i, j] = 0x3F80
        Yu = B.cas_gemm_verify_mx(ctx, mw, _dev(torch, U)).cpu().numpy()
        for i, j in enumerate(picks):
            np.testing.assert_array_equal(Yu[i], O.bf16_to_f64(Wc[:, j]).astype(np.float32))


def test_gemm_verify_mx_gives_a_column_the_same_bits_in_any_company(env):
    torch, B, ctx = env
    rows, cols, keep, t = 150, 1000, 600, 4
    W = _matrix(rows, cols, False, seed=5)
    X = synth.activations(cols, 20, seed=6)
    mw = B.cas_mx_encode(ctx, B.cas_encode_weight(ctx, _dev(torch, W), keep, t))
    Y20 = B.cas_gemm_verify_mx(ctx, mw, _dev(torch, X)).cpu().numpy()
    Y5 = B.cas_gemm_verify_mx(ctx, mw, _dev(torch, X[:5])).cpu().numpy()
    np.testing.assert_array_equal(Y20[:5], Y5)
    for c in (0, 7, 19):
        y1 = B.cas_gemm_verify_mx(ctx, mw, _dev(torch, X[c:c + 1])).cpu().numpy()
        np.testing.assert_array_equal(y1[0], Y20[c])


def test_mx_empty_matrix(env):
    torch, B, ctx = env
    ew = B.cas_encode_weight(ctx, torch.empty((0, 256), dtype=torch.int16, device="cuda"), 600, 4)
    mw = B.cas_mx_encode(ctx, ew)
    assert B.cas_mx_decode(ctx, mw, full=True).shape == (0, 256)
    x = _dev(torch, synth.activations(256, 1, seed=1))
    assert B.cas_gemv_draft_mx(ctx, mw, x).shape == (0,)
