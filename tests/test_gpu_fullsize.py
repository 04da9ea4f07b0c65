"""Parity at the full sizes and launch configuration of the bench (Llama-3-8B layer shapes,
paper-default format): inputs are generated on the GPU as in the bench, sampled output rows are
checked one by one against the oracle (selection, streams, draft GEMV, verify GEMM), plus
properties that hold at any size (kept count per row, exact reconstruction)."""
import numpy as np
import pytest

from oracle import cassandra_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_26558_amd import binding as B
    return torch, B, B.Context()


SHAPES = [(28672, 4096), (4096, 14336), (6144, 4096), (128256, 4096),
          (8192, 28672), (10240, 8192)]     # the last two: Llama-3-70B down and qkv projections


@pytest.mark.parametrize("rows,cols", SHAPES)
def test_sampled_rows_against_oracle(env, rows, cols):
    torch, B, ctx = env
    from paper_2605_26558_amd.workload import _random_weight
    print(f"case rows={rows} cols={cols}", flush=True)
    keep, t, k = 600, 4, 6
    gen = torch.Generator(device="cuda"); gen.manual_seed(rows + cols)
    W = _random_weight(torch, rows, cols, gen)
    act = torch.exp(0.5 * torch.randn(cols, device="cuda", generator=gen))
    X = torch.randn((k + 1, cols), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
    ew = B.cas_encode_weight(ctx, W, keep, t, act)
    d = ew.desc
    yd = B.cas_gemv_draft(ctx, ew, X[:1].contiguous())
    yv = B.cas_gemm_verify(ctx, ew, X)
    # properties at full size: every row keeps exactly K values; reconstruction is exact
    bm = ew.spec[d.off_bitmap: d.off_bitmap + rows * d.bw * 4].view(torch.int32).reshape(rows, d.bw)
    cnt = torch.zeros(rows, dtype=torch.int64, device="cuda")
    for b in range(32):
        cnt += ((bm >> b) & 1).sum(dim=1)
    assert int(cnt.min()) == d.K and int(cnt.max()) == d.K
    full = B.cas_decode_weight(ctx, ew, full=True)
    assert torch.equal(full, W)
    del full
    # sampled rows, one by one, against the oracle
    rng = np.random.default_rng(rows)
    idx = np.unique(np.concatenate([[0, rows - 1], rng.integers(0, rows, 30)]))
    Wh = W[torch.from_numpy(idx).cuda()].cpu().numpy().view(np.uint16)
    ah = act.cpu().numpy()
    Xh = X.cpu().numpy().view(np.uint16)
    p = O.encode_weight(Wh, keep, t, ah)
    sp = ew.spec.cpu().numpy(); vf = ew.verif.cpu().numpy()
    def rowsof(buf, off, w):
        return np.stack([buf[off + r * w * 4: off + (r + 1) * w * 4].view("<u4") for r in idx])
    np.testing.assert_array_equal(rowsof(sp, d.off_bitmap, d.bw), p.bitmap)
    np.testing.assert_array_equal(rowsof(sp, d.off_spec, d.sw), p.spec)
    np.testing.assert_array_equal(rowsof(vf, d.off_lo, d.lw), p.lo)
    np.testing.assert_array_equal(rowsof(vf, d.off_pruned, d.pw), p.pruned)
    wn = np.linalg.norm(O.bf16_to_f64(Wh), axis=1)
    xn = np.linalg.norm(O.bf16_to_f64(Xh), axis=1)
    ed = np.abs(yd.cpu().numpy()[0, idx] - O.gemv_draft(p, Xh[0])) / (wn * xn[0])
    ev = np.abs(yv.cpu().numpy()[:, idx] - O.gemm_verify(p, Xh)) / (wn[None, :] * xn[:, None])
    assert ed.max() < 2e-5 and ev.max() < 2e-5, (ed.max(), ev.max())


def test_attention_at_bench_context_sampled_heads(env):
    """8192 committed positions (synthetic K/V through the online encoder), draft and verify
    attention of one layer against the oracle on the decoded cache."""
    torch, B, _ = env
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    ctx = B.Context(workspace=ws)
    nq, nkv, L = 32, 8, 8192
    kv = B.KVCache(ctx, 1, nkv, n_pages=130, max_seqs=1, max_pages_per_seq=130)
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    K = torch.randn((L, nkv, 128), device="cuda", generator=gen)
    K[:, :, torch.tensor([3, 40, 77, 100])] *= 10.0
    V = torch.randn((L, nkv, 128), device="cuda", generator=gen)
    Kb = K.to(torch.bfloat16).view(torch.int16).contiguous(); Vb = V.to(torch.bfloat16).view(torch.int16).contiguous()
    B.cas_kv_append(ctx, kv, 0, 0, Kb, Vb)
    B.cas_kv_set_len(kv, 0, L)
    Kf, Vf = B.cas_kv_read(ctx, kv, 0, 0, 0, L, full=True)
    assert torch.equal(Kf, Kb) and torch.equal(Vf, Vb)
    Kd, Vd = B.cas_kv_read(ctx, kv, 0, 0, 0, L, full=False)
    for ncols, full in ((1, False), (7, True)):
        Q = (torch.randn((ncols, nq, 128), device="cuda", generator=gen) * 0.3).to(torch.bfloat16).view(torch.int16)
        Kn = torch.randn((ncols, nkv, 128), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
        Vn = torch.randn((ncols, nkv, 128), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
        out = B.cas_attention(ctx, kv, 0, 0, full, Q, Kn, Vn).cpu().numpy().view(np.uint16)
        Kc = (Kf if full else Kd).cpu().numpy().view(np.uint16)
        Vc = (Vf if full else Vd).cpu().numpy().view(np.uint16)
        Qh, Knh, Vnh = (x.cpu().numpy().view(np.uint16) for x in (Q, Kn, Vn))
        for c in (0, ncols - 1):
            vis = c + 1
            kk = O.bf16_to_f64(np.concatenate([Kc, Knh[:vis]])); vv = O.bf16_to_f64(np.concatenate([Vc, Vnh[:vis]]))
            for h in (0, 13, 31):
                q = O.bf16_to_f64(Qh[c, h])
                ref = O.attention_one(q, kk[:, h // 4, :], vv[:, h // 4, :])
                s = kk[:, h // 4, :] @ q / np.sqrt(128.0)
                pr = np.exp(s - s.max()); pr /= pr.sum()
                tol = 2e-3 * np.linalg.norm(pr) * np.linalg.norm(vv[:, h // 4, :], axis=0) + 2.0 ** -8 * np.abs(ref)
                err = np.abs(O.bf16_to_f64(out[c, h]) - ref)
                assert (err <= tol).all(), (ncols, c, h, float((err / tol).max()))
