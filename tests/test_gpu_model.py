"""GPU parity of the model-level steps (draft_step, verify_step, commit, spec_round, prefill)
against the oracle on a small Llama-shaped model, through the C ABI."""
import numpy as np
import pytest

from oracle import cassandra_oracle as O
import synth
from conftest import LOGIT_SLACK, record_ratio

pytestmark = pytest.mark.gpu

SHAPE = synth.TINY
MAX_POS = 128


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2605_26558_amd import binding as B
    ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda")
    return torch, B, B.Context(workspace=ws)


def _dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def gpu_model(torch, B, ctx, weights, keep, t, max_cols, kv_exp_mode=0):
    layers = []
    for lw in weights["layers"]:
        L = {n: B.cas_encode_weight(ctx, _dev(torch, lw[n]), keep, t) for n in ("wqkv", "wo", "wgu", "wd")}
        L["g_attn"], L["g_ffn"] = _dev(torch, lw["g_attn"]), _dev(torch, lw["g_ffn"])
        layers.append(L)
    head = B.cas_encode_weight(ctx, _dev(torch, weights["lm_head"]), keep, t)
    rope = torch.from_numpy(synth.rope_table(MAX_POS, SHAPE.head_dim, SHAPE.rope_theta)).cuda()
    model = B.Model(ctx, SHAPE, layers, head, _dev(torch, weights["embed"]), _dev(torch, weights["g_final"]), rope,
                    max_cols)
    kv = B.KVCache(ctx, SHAPE.n_layers, SHAPE.n_kv_heads, n_pages=2, max_seqs=1, max_pages_per_seq=2,
                   keep_permille=keep, trunc_bits=t, exp_mode=kv_exp_mode)
    return model, kv


def oracle_model(weights, keep, t):
    tab = synth.rope_table(MAX_POS, SHAPE.head_dim, SHAPE.rope_theta)
    return O.OracleModel(SHAPE, weights, tab, w_keep=keep, w_t=t, kv_keep=keep, kv_t=t)


def _logit_tol(om, draft):
    """2e-3 |W_row| |x| of the output head with |x| = |g_final| sqrt(hidden)-ish: the normalised
    hidden state has unit rms before the gain."""
    W = om.W(None, "lm_head", draft)
    xnorm = np.linalg.norm(O.bf16_to_f64(om.g_final))
    return 2e-3 * np.linalg.norm(W, axis=1) * xnorm


def _check_logits(gpu, ref, tol, what):
    err = np.abs(gpu - ref)
    # errors of earlier layers (bf16 roundings that fall differently) also reach the head
    assert (err <= LOGIT_SLACK * tol[None, :]).all(), (what, float((err / tol[None, :]).max()))
    for c in range(ref.shape[0]):
        a, b = int(np.argmax(gpu[c])), int(np.argmax(ref[c]))
        if a != b:
            top2 = np.sort(ref[c])[-2:]
            assert top2[1] - top2[0] <= LOGIT_SLACK * tol.max(), (what, c, a, b, top2)
    return float((err / tol[None, :]).max())


@pytest.mark.parametrize("keep,t", [(600, 4), (250, 4)])
def test_verify_and_draft_steps_match_oracle(env, keep, t):
    torch, B, ctx = env
    weights = synth.model_weights(SHAPE, seed=1)
    model, kv = gpu_model(torch, B, ctx, weights, keep, t, max_cols=8)
    om = oracle_model(weights, keep, t)
    prompt = synth.token_ids(6, SHAPE.vocab, seed=5)
    # verification pass over 6 columns on an empty cache
    toks = torch.from_numpy(prompt).cuda()
    tgt = torch.empty(6, dtype=torch.int32, device="cuda")
    logits = torch.empty((6, SHAPE.vocab), dtype=torch.float32, device="cuda")
    B.cas_verify_step(ctx, model, kv, 0, toks, 5, tgt, logits)
    ref, new_kv = om.forward(prompt, draft=False)
    r = _check_logits(logits.cpu().numpy().astype(np.float64), ref, _logit_tol(om, False), "verify")
    record_ratio(f"tiny_model_verify_logits_keep{keep}", r)
    assert (tgt.cpu().numpy() == np.argmax(logits.cpu().numpy(), axis=1)).all()
    # commit all six, compare the cache contents with the oracle's K/V
    B.cas_commit(ctx, model, kv, 0, 5)
    om.append_kv(new_kv, 6)
    assert B.cas_kv_len(kv, 0) == 6
    for layer in range(SHAPE.n_layers):
        Kf, Vf = B.cas_kv_read(ctx, kv, layer, 0, 0, 6, full=True)
        for got, want in ((Kf, new_kv[layer][0]), (Vf, new_kv[layer][1])):
            g = O.bf16_to_f64(got.cpu().numpy().view(np.uint16)); w = O.bf16_to_f64(want)
            assert np.abs(g - w).max() <= 0.05 * np.abs(w).max()
            assert (np.abs(g - w) > 2.0 ** -7 * np.abs(w) + 1e-3).mean() < 0.02
    # two chained draft passes from the next token
    cur = torch.tensor([int(np.argmax(ref[5]))], dtype=torch.int32, device="cuda")
    extra = [(np.zeros((0, SHAPE.n_kv_heads, 128), np.uint16),) * 2 for _ in range(SHAPE.n_layers)]
    for slot in range(2):
        nxt = torch.empty(1, dtype=torch.int32, device="cuda")
        dl = torch.empty((1, SHAPE.vocab), dtype=torch.float32, device="cuda")
        B.cas_draft_step(ctx, model, kv, 0, cur, slot, nxt, dl)
        oref, okv = om.forward([int(cur.item())], draft=True, extra_kv=extra)
        extra = [(np.concatenate([e[0], n[0]]), np.concatenate([e[1], n[1]])) for e, n in zip(extra, okv)]
        r = _check_logits(dl.cpu().numpy().astype(np.float64), oref, _logit_tol(om, True), f"draft{slot}")
        record_ratio(f"tiny_model_draft{slot}_logits_keep{keep}", r)
        cur = torch.tensor([int(np.argmax(oref[0]))], dtype=torch.int32, device="cuda")   # teacher forcing


def test_model_steps_on_unary_coded_weights(env):
    """Every linear layer switched to the unary form of its speculation data (Sec. 4.2 lossless
    configuration): the verification pass gives the bits of the raw form, the draft pass the
    oracle's logits within the usual tolerance, and a speculative round emits the same tokens."""
    torch, B, ctx = env
    keep, t = 600, 4
    weights = synth.model_weights(SHAPE, seed=1)
    model, kv = gpu_model(torch, B, ctx, weights, keep, t, max_cols=8)
    om = oracle_model(weights, keep, t)
    prompt = synth.token_ids(6, SHAPE.vocab, seed=5)
    toks = torch.from_numpy(prompt).cuda()

    def run():
        B.cas_kv_set_len(kv, 0, 0)
        tgt = torch.empty(6, dtype=torch.int32, device="cuda")
        vl = torch.empty((6, SHAPE.vocab), dtype=torch.float32, device="cuda")
        B.cas_verify_step(ctx, model, kv, 0, toks, 5, tgt, vl)
        B.cas_commit(ctx, model, kv, 0, 5)
        cur = torch.tensor([int(prompt[-1])], dtype=torch.int32, device="cuda")
        nxt = torch.empty(1, dtype=torch.int32, device="cuda")
        dl = torch.empty((1, SHAPE.vocab), dtype=torch.float32, device="cuda")
        B.cas_draft_step(ctx, model, kv, 0, cur, 0, nxt, dl)
        n, emitted = B.cas_spec_round(ctx, model, kv, 0, int(prompt[-1]), 4)
        return vl.cpu().numpy(), tgt.cpu().numpy(), dl.cpu().numpy(), (n, emitted)

    raw = run()
    layers, head = model._keep[0], model._keep[1]
    for l, L in enumerate(layers):
        for which, name in enumerate(("wqkv", "wo", "wgu", "wd")):
            model.use_unary(l, which, B.cas_unary_encode(ctx, L[name]))
    model.use_unary(-1, 0, B.cas_unary_encode(ctx, head))
    una = run()
    np.testing.assert_array_equal(una[0], raw[0])      # verification logits: same kernel, same bits
    np.testing.assert_array_equal(una[1], raw[1])
    # draft logits against the oracle (its draft view is the same for both forms: the re-coding is lossless)
    ref, new_kv = om.forward(prompt, draft=False)
    om.append_kv(new_kv, 6)
    extra = [(np.zeros((0, SHAPE.n_kv_heads, 128), np.uint16),) * 2 for _ in range(SHAPE.n_layers)]
    oref, _ = om.forward([int(prompt[-1])], draft=True, extra_kv=extra)
    r = _check_logits(una[2].astype(np.float64), oref, _logit_tol(om, True), "draft on unary weights")
    record_ratio("tiny_model_draft_logits_unary", r)
    # the round emits the target's greedy stream whatever was drafted: both runs give a prefix of it
    m_ = min(len(una[3][1]), len(raw[3][1]))
    assert una[3][1][:m_] == raw[3][1][:m_]
    # a descriptor of another tensor is refused; switching back restores the raw path
    with pytest.raises(B.CasError):
        model.use_unary(0, 0, model._unary[(0, 1)])
    model.use_unary(-1, 0, None)
    for l in range(len(layers)):
        for which in range(4):
            model.use_unary(l, which, None)
    back = run()
    np.testing.assert_array_equal(back[2], raw[2])


@pytest.mark.parametrize("kv_mx", [False, True])
def test_model_steps_on_shared_exponent_weights(env, kv_mx):
    """Every linear layer in the shared-exponent form (Sec. 4.2, the MX approach): the target is
    the converted model.  Verification and draft logits against the oracle run in that mode;
    kv_mx: the cache in the shared-exponent form as well (the whole "Cassandra-2" configuration)."""
    torch, B, ctx = env
    keep, t = 600, 4
    weights = synth.model_weights(SHAPE, seed=1)
    model, kv = gpu_model(torch, B, ctx, weights, keep, t, max_cols=8, kv_exp_mode=B.CAS_EXP_SHARED if kv_mx else 0)
    layers, head = model._keep[0], model._keep[1]
    for l, L in enumerate(layers):
        for which, name in enumerate(("wqkv", "wo", "wgu", "wd")):
            model.use_mx(l, which, B.cas_mx_encode(ctx, L[name]))
    model.use_mx(-1, 0, B.cas_mx_encode(ctx, head))
    tab = synth.rope_table(MAX_POS, SHAPE.head_dim, SHAPE.rope_theta)
    om = O.OracleModel(SHAPE, weights, tab, w_keep=keep, w_t=t, kv_keep=keep, kv_t=t, exp_mode="mx",
                       kv_exp_mode="mx" if kv_mx else "raw")
    prompt = synth.token_ids(6, SHAPE.vocab, seed=5)
    toks = torch.from_numpy(prompt).cuda()
    tgt = torch.empty(6, dtype=torch.int32, device="cuda")
    vl = torch.empty((6, SHAPE.vocab), dtype=torch.float32, device="cuda")
    B.cas_verify_step(ctx, model, kv, 0, toks, 5, tgt, vl)
    ref, new_kv = om.forward(prompt, draft=False)
    r = _check_logits(vl.cpu().numpy().astype(np.float64), ref, _logit_tol(om, False), "verify, shared exponents")
    record_ratio("tiny_model_verify_logits_mx" + ("_kv" if kv_mx else ""), r)
    B.cas_commit(ctx, model, kv, 0, 5)
    om.append_kv(new_kv, 6)
    cur = torch.tensor([int(np.argmax(ref[5]))], dtype=torch.int32, device="cuda")
    nxt = torch.empty(1, dtype=torch.int32, device="cuda")
    dl = torch.empty((1, SHAPE.vocab), dtype=torch.float32, device="cuda")
    B.cas_draft_step(ctx, model, kv, 0, cur, 0, nxt, dl)
    extra = [(np.zeros((0, SHAPE.n_kv_heads, 128), np.uint16),) * 2 for _ in range(SHAPE.n_layers)]
    oref, _ = om.forward([int(cur.item())], draft=True, extra_kv=extra)
    r = _check_logits(dl.cpu().numpy().astype(np.float64), oref, _logit_tol(om, True), "draft, shared exponents")
    record_ratio("tiny_model_draft_logits_mx" + ("_kv" if kv_mx else ""), r)
    # speculation against the converted model is lossless: the stream of rounds equals plain decoding
    gen_prompt = synth.token_ids(5, SHAPE.vocab, seed=9)
    plain, _ = _gpu_generate(torch, B, ctx, model, kv, gen_prompt, 16, 0)
    spec, stats = _gpu_generate(torch, B, ctx, model, kv, gen_prompt, 16, 4)
    assert spec == plain, (spec, plain)


def _gpu_generate(torch, B, ctx, model, kv, prompt, n_new, k):
    B.cas_kv_set_len(kv, 0, 0)
    if len(prompt) > 1:
        B.cas_prefill(ctx, model, kv, 0, torch.from_numpy(prompt[:-1].copy()).cuda())
    pending, out, stats = int(prompt[-1]), [], []
    while len(out) < n_new:
        n, emitted = B.cas_spec_round(ctx, model, kv, 0, pending, k)
        out.extend(emitted)
        stats.append(n)
        pending = emitted[-1]
    return out[:n_new], stats


@pytest.mark.parametrize("keep,t", [(600, 4), (1000, 0)])
def test_speculative_stream_equals_plain_stream_on_gpu(env, keep, t):
    """Greedy speculative decoding reproduces the target model's stream exactly (Sec. 2.2):
    the verify kernels give a column the same value whatever rides along, so this holds bit
    for bit on the GPU."""
    torch, B, ctx = env
    weights = synth.model_weights(SHAPE, seed=2)
    model, kv = gpu_model(torch, B, ctx, weights, keep, t, max_cols=8)
    prompt = synth.token_ids(20, SHAPE.vocab, seed=6)
    plain, _ = _gpu_generate(torch, B, ctx, model, kv, prompt, 24, 0)
    for k in (1, 4, 7):
        spec, stats = _gpu_generate(torch, B, ctx, model, kv, prompt, 24, k)
        assert spec == plain, (k, spec, plain)
        assert all(0 <= n <= k for n in stats)
        if keep == 1000 and t == 0:
            assert all(n == k for n in stats)          # the draft model is the target model
        print(f"k={k} accepted per round {stats}", flush=True)


def test_gpu_stream_against_oracle_teacher_forced(env):
    """Each GPU target token equals the oracle's unless the oracle's own top-2 margin is inside
    the floating-point tolerance of the logits."""
    torch, B, ctx = env
    keep, t = 600, 4
    weights = synth.model_weights(SHAPE, seed=3)
    model, kv = gpu_model(torch, B, ctx, weights, keep, t, max_cols=8)
    om = oracle_model(weights, keep, t)
    prompt = synth.token_ids(5, SHAPE.vocab, seed=7)
    B.cas_prefill(ctx, model, kv, 0, torch.from_numpy(prompt[:-1].copy()).cuda())
    pending = O.prefill(om, prompt)
    tol = _logit_tol(om, False)
    excused = 0
    for step in range(10):
        ref, okv = om.forward([pending], draft=False)
        om.append_kv(okv, 1)
        tok = torch.tensor([pending], dtype=torch.int32, device="cuda")
        tgt = torch.empty(1, dtype=torch.int32, device="cuda")
        B.cas_verify_step(ctx, model, kv, 0, tok, 0, tgt, None)
        B.cas_commit(ctx, model, kv, 0, 0)
        want = O.argmax_lowest(ref[0])
        got = int(tgt.item())
        if got != want:
            top2 = np.sort(ref[0])[-2:]
            assert top2[1] - top2[0] <= LOGIT_SLACK * tol.max(), (step, got, want)
            excused += 1
        pending = want
    print("excused near-ties:", excused, flush=True)
    assert excused <= 2


def test_multi_sequence_passes_equal_single_sequence_passes(env):
    """Draft and verification passes over several sequences at once give every sequence exactly
    the tokens, and after the commit exactly the cache contents, of the one-sequence calls:
    a column's value never depends on what rides along."""
    torch, B, ctx = env
    keep, t, k, nseq = 600, 4, 3, 3
    weights = synth.model_weights(SHAPE, seed=4)
    layers = []
    for lw in weights["layers"]:
        L = {n: B.cas_encode_weight(ctx, _dev(torch, lw[n]), keep, t) for n in ("wqkv", "wo", "wgu", "wd")}
        L["g_attn"], L["g_ffn"] = _dev(torch, lw["g_attn"]), _dev(torch, lw["g_ffn"])
        layers.append(L)
    head = B.cas_encode_weight(ctx, _dev(torch, weights["lm_head"]), keep, t)
    rope = torch.from_numpy(synth.rope_table(MAX_POS, SHAPE.head_dim, SHAPE.rope_theta)).cuda()
    model = B.Model(ctx, SHAPE, layers, head, _dev(torch, weights["embed"]), _dev(torch, weights["g_final"]), rope,
                    max_cols=12, max_seqs=nseq)
    def cache():
        return B.KVCache(ctx, SHAPE.n_layers, SHAPE.n_kv_heads, n_pages=2 * nseq, max_seqs=nseq, max_pages_per_seq=2,
                         keep_permille=keep, trunc_bits=t)
    kv_a, kv_b = cache(), cache()
    prompts = [synth.token_ids(n, SHAPE.vocab, seed=20 + n) for n in (10, 37, 70)]
    for kv in (kv_a, kv_b):
        for s, p in enumerate(prompts):
            B.cas_prefill(ctx, model, kv, s, torch.from_numpy(p[:-1].copy()).cuda())
    # one sequence at a time
    single = []
    for s, p in enumerate(prompts):
        tok = torch.zeros(k + 1, dtype=torch.int32, device="cuda"); tok[0] = int(p[-1])
        tgt = torch.zeros(k + 1, dtype=torch.int32, device="cuda")
        for i in range(k):
            B.cas_draft_step(ctx, model, kv_a, s, tok[i:i + 1], i, tok[i + 1:i + 2])
        B.cas_verify_step(ctx, model, kv_a, s, tok, k, tgt)
        B.cas_commit(ctx, model, kv_a, s, 2)
        single.append((tok.cpu().numpy().copy(), tgt.cpu().numpy().copy()))
    # all sequences per pass
    toks = torch.zeros((k + 1, nseq), dtype=torch.int32, device="cuda")
    toks[0] = torch.tensor([int(p[-1]) for p in prompts], dtype=torch.int32)
    for i in range(k):
        B.cas_draft_step_multi(ctx, model, kv_b, list(range(nseq)), [i] * nseq, toks[i], toks[i + 1])
    cols = toks.t().contiguous().reshape(-1)                 # sequence after sequence
    tgt = torch.zeros(nseq * (k + 1), dtype=torch.int32, device="cuda")
    B.cas_verify_step_multi(ctx, model, kv_b, list(range(nseq)), [k] * nseq, cols, tgt)
    for s in range(nseq):
        B.cas_commit(ctx, model, kv_b, s, 2)
    cols_h, tgt_h = cols.cpu().numpy().reshape(nseq, k + 1), tgt.cpu().numpy().reshape(nseq, k + 1)
    for s in range(nseq):
        np.testing.assert_array_equal(cols_h[s], single[s][0])
        np.testing.assert_array_equal(tgt_h[s], single[s][1])
        n = B.cas_kv_len(kv_a, s)
        assert n == B.cas_kv_len(kv_b, s) == len(prompts[s]) - 1 + 3
        for layer in range(SHAPE.n_layers):
            Ka, Va = B.cas_kv_read(ctx, kv_a, layer, s, 0, n, full=True)
            Kb, Vb = B.cas_kv_read(ctx, kv_b, layer, s, 0, n, full=True)
            assert torch.equal(Ka, Kb) and torch.equal(Va, Vb)


@pytest.mark.parametrize("max_cols,k,nseq,form", [(12, 3, 3, "raw"), (8, 3, 3, "raw"), (4, 3, 3, "raw"),
                                                  (20, 4, 4, "raw"), (32, 7, 4, "raw"),
                                                  (12, 3, 3, "unary"), (20, 4, 4, "unary"),
                                                  (12, 3, 3, "mx"), (20, 4, 4, "mx")])
def test_multi_sequence_round_equals_single_sequence_rounds(env, max_cols, k, nseq, form):
    """cas_spec_round_multi emits, sequence by sequence, the stream cas_spec_round emits, also
    when the verification columns of the sequences need two or three passes, and when one pass
    carries more than 16 columns (20 and 32: the second column block of the verify GEMM).
    form: the exponents of every linear layer raw, unary-coded, or shared (then the cache has
    shared exponents as well)."""
    torch, B, ctx = env
    print(f"case max_cols={max_cols} k={k} nseq={nseq} form={form}", flush=True)
    keep, t = 600, 4
    weights = synth.model_weights(SHAPE, seed=2)
    model, _ = gpu_model(torch, B, ctx, weights, keep, t, max_cols=12)
    # same weights, room for three sequences
    layers, head, embed, g_final, rope = model._keep
    model = B.Model(ctx, SHAPE, layers, head, embed, g_final, rope, max_cols=max_cols, max_seqs=nseq)
    if form != "raw":
        recode = B.cas_unary_encode if form == "unary" else B.cas_mx_encode
        use = model.use_unary if form == "unary" else model.use_mx
        for l, L in enumerate(layers):
            for which, name in enumerate(("wqkv", "wo", "wgu", "wd")):
                use(l, which, recode(ctx, L[name]))
        use(-1, 0, recode(ctx, head))
    def cache():
        return B.KVCache(ctx, SHAPE.n_layers, SHAPE.n_kv_heads, n_pages=2 * nseq, max_seqs=nseq, max_pages_per_seq=2,
                         keep_permille=keep, trunc_bits=t,
                         exp_mode=B.CAS_EXP_SHARED if form == "mx" else B.CAS_EXP_RAW)
    kv_a, kv_b = cache(), cache()
    prompts = [synth.token_ids(n, SHAPE.vocab, seed=40 + n) for n in (5, 20, 33, 11)[:nseq]]
    for kv in (kv_a, kv_b):
        for s, p in enumerate(prompts):
            B.cas_prefill(ctx, model, kv, s, torch.from_numpy(p[:-1].copy()).cuda())
    rounds = 5
    single = []
    for s, p in enumerate(prompts):
        pending, out = int(p[-1]), []
        for _ in range(rounds):
            n, emitted = B.cas_spec_round(ctx, model, kv_a, s, pending, k)
            out.append((n, emitted)); pending = emitted[-1]
        single.append(out)
    pending = [int(p[-1]) for p in prompts]
    multi = [[] for _ in range(nseq)]
    for _ in range(rounds):
        res = B.cas_spec_round_multi(ctx, model, kv_b, list(range(nseq)), pending, k)
        for s, (n, emitted) in enumerate(res):
            multi[s].append((n, emitted)); pending[s] = emitted[-1]
    assert multi == single
    for s in range(nseq):
        assert B.cas_kv_len(kv_a, s) == B.cas_kv_len(kv_b, s)


def test_step_calls_replay_from_a_hip_graph():
    """cas_draft_step and cas_verify_step enqueue kernels only (no copies, no memsets), so a
    caller may capture them.  A graph holding one draft pass and one 4-column verification pass
    is replayed three times with other work and synchronisations in between; every replay gives
    the bits of the eager calls.  (The cache length is an argument of the kernels: a graph stays
    valid for the cache state it was captured in.)"""
    import torch
    from paper_2605_26558_amd import binding as B
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx = B.Context(workspace=torch.empty(32 << 20, dtype=torch.uint8, device="cuda"))
        weights = synth.model_weights(SHAPE, seed=4)
        model, kv = gpu_model(torch, B, ctx, weights, 600, 4, max_cols=8)
        prompt = synth.token_ids(20, SHAPE.vocab, seed=6)
        B.cas_prefill(ctx, model, kv, 0, torch.from_numpy(prompt).cuda())
        tok = torch.tensor([5], dtype=torch.int32, device="cuda")
        toks4 = torch.tensor([5, 9, 2, 7], dtype=torch.int32, device="cuda")
        nxt = torch.empty(1, dtype=torch.int32, device="cuda")
        dl = torch.empty((1, SHAPE.vocab), dtype=torch.float32, device="cuda")
        tgt = torch.empty(4, dtype=torch.int32, device="cuda")
        vl = torch.empty((4, SHAPE.vocab), dtype=torch.float32, device="cuda")

        def steps():
            B.cas_draft_step(ctx, model, kv, 0, tok, 0, nxt, dl)
            B.cas_verify_step(ctx, model, kv, 0, toks4, 3, tgt, vl)
        steps()                                  # eager: also grants the kernels their LDS sizes
        side.synchronize()
        want = [t.clone() for t in (nxt, dl, tgt, vl)]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps()
        for rep in range(3):
            for t in (nxt, dl, tgt, vl):
                t.zero_()
            scratch = torch.randn(1 << 20, device="cuda").sum()      # unrelated eager work between replays
            side.synchronize()
            graph.replay()
            side.synchronize()
            for got, ref in zip((nxt, dl, tgt, vl), want):
                assert torch.equal(got, ref), rep
            assert bool(torch.isfinite(scratch))
    torch.cuda.synchronize()


def test_plain_bf16_baseline_step_matches_the_oracles_target_pass(env):
    """cas_dense_decode_step (uncompressed weights, uncompressed cache: the BFloat16 baseline) run
    token by token gives the logits of the oracle's target pass, which is exact bf16 decoding
    (Sec. 4.1: the verification data restore the original model bit for bit)."""
    torch, B, ctx = env
    keep, t = 600, 4
    weights = synth.model_weights(SHAPE, seed=1)
    model, kv = gpu_model(torch, B, ctx, weights, keep, t, max_cols=8)
    om = oracle_model(weights, keep, t)
    dense = [{n: _dev(torch, lw[n]) for n in ("wqkv", "wo", "wgu", "wd")} for lw in weights["layers"]]
    head = _dev(torch, weights["lm_head"])
    kvd = SHAPE.n_kv_heads * SHAPE.head_dim
    kc = torch.zeros((SHAPE.n_layers, MAX_POS, kvd), dtype=torch.int16, device="cuda")
    vc = torch.zeros_like(kc)
    tokens = synth.token_ids(70, SHAPE.vocab, seed=13)          # crosses a page of 64 positions
    tol = _logit_tol(om, False)
    worst = 0.0
    for i, tok in enumerate(tokens):
        tin = torch.tensor([int(tok)], dtype=torch.int32, device="cuda")
        tout = torch.empty(1, dtype=torch.int32, device="cuda")
        lg = torch.empty((1, SHAPE.vocab), dtype=torch.float32, device="cuda")
        B.cas_dense_decode_step(ctx, model, dense, head, kc, vc, i, tin, tout, lg)
        ref, new_kv = om.forward([int(tok)], draft=False)
        om.append_kv(new_kv, 1)
        got = lg.cpu().numpy().astype(np.float64)
        worst = max(worst, _check_logits(got, ref, tol, f"dense step {i}"))
        assert int(tout[0]) == int(np.argmax(got[0]))
        if i in (0, 63, 69):   # the rows the step stored are the oracle's k, v of that position
            for layer in range(SHAPE.n_layers):
                k_ref = new_kv[layer][0][0].reshape(-1)
                k_got = kc[layer, i].cpu().numpy().view(np.uint16)
                d = np.abs(O.bf16_to_f64(k_got) - O.bf16_to_f64(k_ref))
                assert d.max() <= 0.05 * np.abs(O.bf16_to_f64(k_ref)).max()
    record_ratio("tiny_model_plain_bf16_baseline_logits", worst)
