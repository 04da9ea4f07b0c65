"""GPU parity of the unary-exponent form of the speculation data (Sec. 4.2 exponent
compression) against the oracle, through the C ABI: every region of the buffer bit for bit,
both reconstructions, the draft GEMV and the verification GEMM read from the unary form."""
import numpy as np
import pytest

from oracle import cassandra_oracle as O
import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_26558_amd import binding as B
    ws = torch.empty(8 << 20, dtype=torch.uint8, device="cuda")
    return torch, B, B.Context(workspace=ws)


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def _regions(uw):
    u, d = uw.desc, uw.desc.base
    b = uw.uspec.cpu().numpy()
    def words(off, n):
        return b[off: off + 4 * n].view("<u4")
    return (words(u.off_bitmap, d.rows * d.bw).reshape(d.rows, d.bw),
            words(u.off_sm, d.rows * u.smw).reshape(d.rows, u.smw),
            b[u.off_table: u.off_table + 512].copy(),
            words(u.off_rowoff, d.rows + 1),
            words(u.off_ue, u.ue_words))


CASES = [
    # rows, cols, keep, t, special values
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
    W = synth.weight_matrix(rows, cols, seed=seed)
    if special:   # rare exponents (long codes that cross several words), zeros, Inf, NaN
        rng = np.random.Generator(np.random.Philox(seed + 1))
        idx = rng.integers(0, W.size, size=min(W.size, 64))
        W.reshape(-1)[idx] = rng.integers(0, 65536, size=idx.shape).astype(np.uint16)
        W.reshape(-1)[idx[:4]] = np.array([0x7F80, 0xFFFF, 0x0001, 0x8000], dtype=np.uint16)[: len(idx[:4])]
    return W


@pytest.mark.parametrize("rows,cols,keep,t,special", CASES)
def test_unary_buffer_and_reconstruction_bit_exact(env, rows, cols, keep, t, special):
    torch, B, ctx = env
    print(f"case rows={rows} cols={cols} keep={keep} t={t} special={special}", flush=True)
    W = _matrix(rows, cols, special, seed=rows + cols + t)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), keep, t)
    uw = B.cas_unary_encode(ctx, ew)
    torch.cuda.synchronize()
    p = O.encode_weight(W, keep, t)
    u = O.to_unary(p)
    assert uw.desc.ue_words == len(u.ue) and uw.desc.smw == u.sm.shape[1]
    np.testing.assert_array_equal(np.frombuffer(bytes(uw.desc.exp_of_rank), dtype=np.uint8), u.exp_of_rank)
    bm, sm, table, rowoff, ue = _regions(uw)
    np.testing.assert_array_equal(bm, p.bitmap)
    np.testing.assert_array_equal(sm, u.sm)
    np.testing.assert_array_equal(table[:256], u.exp_of_rank)
    np.testing.assert_array_equal(table[256:][u.exp_of_rank], np.arange(256, dtype=np.uint8))
    np.testing.assert_array_equal(rowoff, u.ue_off)
    np.testing.assert_array_equal(ue, u.ue)
    full = B.cas_unary_decode(ctx, uw, full=True).cpu().numpy().view(np.uint16)
    draft = B.cas_unary_decode(ctx, uw, full=False).cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(full, W)
    np.testing.assert_array_equal(draft, O.decode_draft(p))


@pytest.mark.parametrize("rows,cols,keep,t,special", [c for c in CASES if not c[4]])
def test_gemv_draft_unary_matches_oracle(env, rows, cols, keep, t, special):
    torch, B, ctx = env
    print(f"case rows={rows} cols={cols} keep={keep} t={t}", flush=True)
    W = _matrix(rows, cols, False, seed=rows + cols + t)
    x = synth.activations(cols, 1, seed=11)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), keep, t)
    uw = B.cas_unary_encode(ctx, ew)
    y = B.cas_gemv_draft_unary(ctx, uw, _dev(torch, x)).cpu().numpy()
    ref = O.gemv_draft_unary(O.to_unary(O.encode_weight(W, keep, t)), x[0])
    tol = np.linalg.norm(O.bf16_to_f64(W), axis=1) * np.linalg.norm(O.bf16_to_f64(x[0])) + 1e-30
    err = np.abs(y - ref) / tol
    assert err.max() < 2e-3          # spec bar
    assert err.max() < 2e-5, err.max()
    # same values as the raw-exponent kernel up to the order of the fp32 sums
    y_raw = B.cas_gemv_draft(ctx, ew, _dev(torch, x)).cpu().numpy()[0]
    assert (np.abs(y - y_raw) / tol).max() < 2e-5


@pytest.mark.parametrize("ncols", [1, 5, 20])
@pytest.mark.parametrize("rows,cols,keep,t,special", [c for c in CASES if not c[4]])
def test_gemm_verify_unary_is_exact_and_equal_to_the_raw_form(env, rows, cols, keep, t, special, ncols):
    """Verification from the unary form (Sec. 4.2 lossless configuration, Sec. 4.1 target
    inference): against the oracle's product with the matrix its unary reconstruction returns,
    and bit for bit against the raw-exponent verification GEMM."""
    torch, B, ctx = env
    print(f"case rows={rows} cols={cols} keep={keep} t={t} ncols={ncols}", flush=True)
    W = _matrix(rows, cols, False, seed=rows + cols + t)
    X = synth.activations(cols, ncols, seed=13)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), keep, t)
    uw = B.cas_unary_encode(ctx, ew)
    Y = B.cas_gemm_verify_unary(ctx, uw, _dev(torch, X)).cpu().numpy()
    u = O.to_unary(O.encode_weight(W, keep, t))
    Wf = O.bf16_to_f64(O.decode_full_unary(u))
    ref = (Wf @ O.bf16_to_f64(X).T).T
    tol = np.linalg.norm(Wf, axis=1)[None, :] * np.linalg.norm(O.bf16_to_f64(X), axis=1)[:, None] + 1e-30
    err = np.abs(Y - ref) / tol
    assert err.max() < 2e-3          # spec bar
    assert err.max() < 2e-5, err.max()
    np.testing.assert_array_equal(Y, B.cas_gemm_verify(ctx, ew, _dev(torch, X)).cpu().numpy())


def test_gemm_verify_unary_in_row_blocks_and_without_room(env):
    """A workspace that holds 16 rows of the raw stream at a time gives the same bits as one that
    holds the matrix; one that holds fewer is refused."""
    torch, B, ctx = env
    rows, cols, keep, t = 150, 1000, 600, 4
    W = _matrix(rows, cols, False, seed=5)
    X = synth.activations(cols, 3, seed=6)
    ew = B.cas_encode_weight(ctx, _dev(torch, W), keep, t)
    uw = B.cas_unary_encode(ctx, ew)
    whole = B.cas_gemm_verify_unary(ctx, uw, _dev(torch, X)).cpu().numpy()
    row_bytes = ew.desc.sw * 4
    small = B.Context(workspace=torch.empty(17 * row_bytes + 256, dtype=torch.uint8, device="cuda"))
    # the matrix itself comes from the first context: buffers are plain device memory
    np.testing.assert_array_equal(B.cas_gemm_verify_unary(small, uw, _dev(torch, X)).cpu().numpy(), whole)
    tiny = B.Context(workspace=torch.empty(15 * row_bytes + 256, dtype=torch.uint8, device="cuda"))
    with pytest.raises(B.CasError) as e:
        B.cas_gemm_verify_unary(tiny, uw, _dev(torch, X))
    assert e.value.code == B.CAS_ENOMEM


def test_unary_empty_matrix(env):
    torch, B, ctx = env
    ew = B.cas_encode_weight(ctx, torch.empty((0, 256), dtype=torch.int16, device="cuda"), 600, 4)
    uw = B.cas_unary_encode(ctx, ew)
    assert uw.desc.ue_words == 0
    assert B.cas_unary_decode(ctx, uw, full=True).shape == (0, 256)
    x = _dev(torch, synth.activations(256, 1, seed=1))
    assert B.cas_gemv_draft_unary(ctx, uw, x).shape == (0,)


def test_unary_plan_and_encode_are_reproducible_on_many_rows(env):
    """More row workgroups than the chip holds at once: every plan of the same matrix reports
    the same codebook and stream size, every encoding the same bytes, and the exact
    reconstruction returns the matrix."""
    torch, B, ctx = env
    rows, cols = 6000, 1024
    gen = torch.Generator(device="cuda"); gen.manual_seed(9)
    W = (torch.randn((rows, cols), device="cuda", generator=gen) * 0.02).to(torch.bfloat16).view(torch.int16)
    ew = B.cas_encode_weight(ctx, W, 600, 4)
    u0 = B.cas_unary_plan(ctx, ew)
    first = B.cas_unary_encode(ctx, ew, u0)
    for _ in range(10):
        u = B.cas_unary_plan(ctx, ew)
        assert u.ue_words == u0.ue_words and bytes(u.exp_of_rank) == bytes(u0.exp_of_rank)
    for _ in range(3):
        again = B.cas_unary_encode(ctx, ew)
        assert torch.equal(again.uspec, first.uspec)
    assert torch.equal(B.cas_unary_decode(ctx, first, full=True), W)
    mx0 = B.cas_mx_encode(ctx, ew)
    for _ in range(3):
        mx = B.cas_mx_encode(ctx, ew)
        assert torch.equal(mx.spec, mx0.spec) and torch.equal(mx.verif, mx0.verif)
