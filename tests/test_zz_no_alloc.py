"""cas_attention_static (the entry point for callers that cannot allocate: partial results in the
library's own fixed device array) gives bit for bit the output of cas_attention, on two calls in
a row of which the second is smaller, and refuses a call whose partials exceed the array."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def test_static_scratch_attention_equals_workspace_attention():
    import torch
    from paper_2605_26558_amd import binding as B
    nq, nkv = 32, 8
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    ctx_ws = B.Context(workspace=ws)
    ctx_none = B.Context()                                  # no workspace at all
    L1, L2 = 2500, 700                                      # 40 and 11 pages: several splits, ragged tails
    kv = B.KVCache(ctx_ws, 1, nkv, n_pages=96, max_seqs=2, max_pages_per_seq=48)
    for seq, (L, seed) in enumerate(((L1, 31), (L2, 41))):
        K = synth.kv_tensor(L, nkv, 128, seed=seed, outlier_channels=4)
        V = synth.kv_tensor(L, nkv, 128, seed=seed + 1, outlier_channels=0)
        B.cas_kv_append(ctx_ws, kv, 0, seq, _dev(torch, K), _dev(torch, V))
        B.cas_kv_set_len(kv, seq, L)
    cases = [(0, True, 7, 7), (1, False, 1, 3)]            # (sequence, full, columns, in-flight): second call smaller
    outs = []
    for seq, full, ncols, n_new in cases:
        Q = _dev(torch, synth.normal_bf16((ncols, nq, 128), 0.3, seed=50 + seq))
        Kn = _dev(torch, synth.kv_tensor(n_new, nkv, 128, seed=60 + seq))
        Vn = _dev(torch, synth.kv_tensor(n_new, nkv, 128, seed=70 + seq, outlier_channels=0))
        want = B.cas_attention(ctx_ws, kv, 0, seq, full, Q, Kn, Vn)
        got = torch.full_like(want, 0x7FC0)
        print(f"static call seq={seq} full={full} ncols={ncols} n_new={n_new}", flush=True)
        B.cas_attention_static(ctx_none, kv, 0, seq, full, Q, Kn, Vn, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (seq, full)
        outs.append((Q, Kn, Vn, want))
    # the first call again after the smaller one: stale records of other calls do not leak in
    Q, Kn, Vn, want = outs[0]
    got = torch.full_like(want, 0x7FC0)
    B.cas_attention_static(ctx_none, kv, 0, 0, True, Q, Kn, Vn, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    # the plain entry point without a workspace is an error, not a fault
    with pytest.raises(B.CasError):
        B.cas_attention(ctx_none, kv, 0, 0, True, Q, Kn, Vn)


def test_static_scratch_rejects_calls_beyond_its_capacity():
    import torch
    from paper_2605_26558_amd import binding as B
    cap = B.cas_attention_static_capacity()
    assert cap == 32 << 20
    nq, nkv, ncols = 32, 8, 16                              # 64 query rows per kv head
    per_split = nkv * ncols * (nq // nkv) * 132 * 4
    pages = cap // per_split + 2                            # partials of this length do not fit
    ctx = B.Context()
    kv = B.KVCache(ctx, 1, nkv, n_pages=1, max_seqs=1, max_pages_per_seq=pages,
                   page_table=torch.zeros((1, pages), dtype=torch.int32))
    B.cas_kv_set_len(kv, 0, (pages - 1) * 64)               # host-side length only: the call must fail before any launch
    Q = torch.zeros((ncols, nq, 128), dtype=torch.int16, device="cuda")
    Kn = torch.zeros((ncols, nkv, 128), dtype=torch.int16, device="cuda")
    out = torch.zeros_like(Q)
    with pytest.raises(B.CasError) as e:
        B.cas_attention_static(ctx, kv, 0, 0, True, Q, Kn, Kn, out)
    assert e.value.code == B.CAS_ENOMEM
