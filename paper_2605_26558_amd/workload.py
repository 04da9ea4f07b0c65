"""Synthetic Llama-3-shaped workload for bench.py: random-init weights generated on the GPU
with the outlier structure of the configs (N(0, 0.02^2), 0.5 % of input columns x20), encoded
into the Cassandra format by the HIP encoder, and the per-round launch sequence."""
from __future__ import annotations

import synth


def _random_weight(torch, rows, cols, gen, sigma=0.02, outlier_frac=0.005, outlier_scale=20.0):
    w = torch.randn((rows, cols), device="cuda", dtype=torch.float32, generator=gen) * sigma
    n_out = int(round(outlier_frac * cols))
    if n_out:
        idx = torch.randperm(cols, device="cuda", generator=gen)[:n_out]
        w[:, idx] *= outlier_scale
    return w.to(torch.bfloat16).view(torch.int16)


class LinearRoundWorkload:
    """All linear layers of the model: k draft passes + one verify pass per step."""

    def __init__(self, B, args, dev):
        import torch
        self.torch, self.B = torch, B
        self.ctx = B.Context()
        self.k = args.k
        shape = synth.LLAMA3_8B
        self.shape = shape
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1234)
        dims = [("wqkv", shape.q_dim + 2 * shape.kv_dim, shape.hidden), ("wo", shape.hidden, shape.q_dim),
                ("wgu", 2 * shape.ffn, shape.hidden), ("wd", shape.hidden, shape.ffn)]
        self.mats = []
        for _ in range(args.layers):
            for name, r, c in dims:
                act = torch.exp(0.5 * torch.randn(c, device="cuda", generator=gen))
                self.mats.append(B.cas_encode_weight(self.ctx, _random_weight(torch, r, c, gen), args.keep,
                                                     args.trunc, act))
        act = torch.exp(0.5 * torch.randn(shape.hidden, device="cuda", generator=gen))
        self.mats.append(B.cas_encode_weight(self.ctx, _random_weight(torch, shape.vocab, shape.hidden, gen),
                                             args.keep, args.trunc, act))
        torch.cuda.synchronize()
        maxc = max(m.desc.cols for m in self.mats)
        maxr = max(m.desc.rows for m in self.mats)
        self.x = {c: torch.randn((self.k + 1, c), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
                  for c in {m.desc.cols for m in self.mats}}
        self.x1 = {c: v[:1].contiguous() for c, v in self.x.items()}
        self.y = torch.empty((self.k + 1, maxr), device="cuda", dtype=torch.float32)
        self.draft_bytes = sum(m.desc.rows * (m.desc.bw + m.desc.sw) * 4 for m in self.mats)
        self.verify_bytes = sum(m.desc.rows * (m.desc.bw + m.desc.sw + m.desc.lw + m.desc.pw) * 4
                                for m in self.mats)
        self.values = sum(m.desc.rows * m.desc.cols for m in self.mats)
        self.bytes_per_step = self.k * self.draft_bytes + self.verify_bytes
        self.config = {"workload": f"Llama-3-8B-shaped linear layers ({args.layers} layers + output head, "
                                   f"{self.values / 1e9:.2f} G weights), batch 1, draft length k={self.k}",
                       "keep_permille": args.keep, "trunc_bits": args.trunc, "k": self.k,
                       "rows_of_hot_path": "weight path only (draft decode+GEMV, verify reconstruct+GEMM)"}

    def _draft_pass(self):
        B, ctx = self.B, self.ctx
        for m in self.mats:
            B.cas_gemv_draft(ctx, m, self.x1[m.desc.cols], self.y[:1, : m.desc.rows])

    def _verify_pass(self):
        B, ctx = self.B, self.ctx
        for m in self.mats:
            B.cas_gemm_verify(ctx, m, self.x[m.desc.cols], self.y[:, : m.desc.rows])

    def step(self):
        for _ in range(self.k):
            self._draft_pass()
        self._verify_pass()

    def _timed(self, fn):
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3

    def roofline_pass(self):
        td = self._timed(self._draft_pass)
        self.t_draft = td
        self.t_verify = self._timed(self._verify_pass)
        n = len(self.mats)
        ach = self.draft_bytes / td / 1e9
        return {"bound": "hbm", "kernel": "gemv_draft_kernel", "achieved": ach, "peak": 8000.0, "unit": "GB/s",
                "frac": ach / 8000.0, "traffic": None,
                "launches": n, "avg_launch_us": td / n * 1e6, "bytes_per_launch": self.draft_bytes / n}

    def extra(self, ms_per_step):
        return {
            "draft_pass_ms": self.t_draft * 1e3, "verify_pass_ms": self.t_verify * 1e3,
            "draft_GBps": self.draft_bytes / self.t_draft / 1e9,
            "verify_GBps": self.verify_bytes / self.t_verify / 1e9,
            "verify_frac_of_peak": self.verify_bytes / self.t_verify / 1e9 / 8000.0,
        }


class ModelRoundWorkload:
    """Whole model: one speculative round (k draft passes, verification over k+1 columns,
    greedy acceptance, commit with online KV encoding) per step, at a fixed context length.
    The cache is pre-filled with synthetic K/V (keys with 4 outlier channels per head x10)
    through the library's online encoder."""

    def __init__(self, B, args, dev):
        import torch
        self.torch, self.B = torch, B
        self.k, self.ctx_len = args.k, args.context
        self.batch = max(1, int(getattr(args, "batch", 1)))
        if self.batch > 4:
            raise SystemExit("--batch: at most 4 sequences")
        big = getattr(args, "model", "8b") == "70b"
        if big:   # hidden 8192, 64 q / 8 kv heads, FFN 28672: ~148 GB encoded at 80 layers
            shape = synth.LlamaShape("llama3-70b", 8192, args.layers, 64, 8, 128, 28672, 128256)
        else:
            shape = synth.LlamaShape("llama3-8b", 4096, args.layers, 32, 8, 128, 14336, 128256)
        self.shape = shape
        name = "Llama-3-70B" if big else "Llama-3-8B"
        # attention partials of the (up to four) sequences that share a launch: one (max, sum,
        # output) record of 132 floats per page, kv head and query row
        rows = (args.k + 1) * (shape.n_q_heads // shape.n_kv_heads)
        pages_ws = (args.context + 1024 + 63) // 64 + 1
        need = min(self.batch, 4) * (pages_ws * shape.n_kv_heads * rows * 132 * 4 + 256)
        self.ws = torch.empty(max(64 << 20, need), dtype=torch.uint8, device="cuda")
        self.ctx = B.Context(workspace=self.ws)
        ctx = self.ctx
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1234)
        dims = {"wqkv": (shape.q_dim + 2 * shape.kv_dim, shape.hidden), "wo": (shape.hidden, shape.q_dim),
                "wgu": (2 * shape.ffn, shape.hidden), "wd": (shape.hidden, shape.ffn)}

        self.dense = []  # plain bf16 copies, only for the vendor-GEMV context figure

        def enc(r, c):
            act = torch.exp(0.5 * torch.randn(c, device="cuda", generator=gen))
            w = _random_weight(torch, r, c, gen)
            if not big:   # the dense copies of the larger model would not fit beside the encoded ones
                self.dense.append(w.view(torch.bfloat16))
            return B.cas_encode_weight(ctx, w, args.keep, args.trunc, act)

        def gain():
            return (1.0 + 0.1 * torch.randn(shape.hidden, device="cuda", generator=gen)).to(torch.bfloat16).view(
                torch.int16)

        layers = []
        for _ in range(shape.n_layers):
            L = {n: enc(r, c) for n, (r, c) in dims.items()}
            L["g_attn"], L["g_ffn"] = gain(), gain()
            layers.append(L)
        head = enc(shape.vocab, shape.hidden)
        embed = torch.randn((shape.vocab, shape.hidden), device="cuda", generator=gen).to(torch.bfloat16).view(
            torch.int16)
        max_pos = self.ctx_len + 1024
        rope = torch.from_numpy(synth.rope_table(max_pos, shape.head_dim, shape.rope_theta)).cuda()
        self.layers, self.head, self.g_final = layers, head, gain()
        nb = self.batch
        # 32 columns per verification pass at most; more sequences x drafts take a second pass
        self.model = B.Model(ctx, shape, layers, head, embed, self.g_final, rope,
                             max_cols=min(32, nb * (self.k + 1)), max_seqs=nb)
        pages = (max_pos + 63) // 64
        kv_mx = getattr(args, "kv_exp_mode", "raw") == "shared"
        self.kv = B.KVCache(ctx, shape.n_layers, shape.n_kv_heads, n_pages=pages * nb, max_seqs=nb,
                            max_pages_per_seq=pages, keep_permille=args.keep, trunc_bits=args.trunc,
                            exp_mode=B.CAS_EXP_SHARED if kv_mx else B.CAS_EXP_RAW)
        # synthetic cache contents
        chunk = 1024
        for layer in range(shape.n_layers):
            out_idx = torch.randperm(128, device="cuda", generator=gen)[:4]
            done = 0
            while done < self.ctx_len:
                n = min(chunk, self.ctx_len - done)
                for seq in range(nb):
                    K = torch.randn((n, shape.n_kv_heads, 128), device="cuda", generator=gen)
                    K[:, :, out_idx] *= 10.0
                    V = torch.randn((n, shape.n_kv_heads, 128), device="cuda", generator=gen)
                    B.cas_kv_set_len(self.kv, seq, done)
                    B.cas_kv_append(ctx, self.kv, layer, seq, K.to(torch.bfloat16).view(torch.int16).contiguous(),
                                    V.to(torch.bfloat16).view(torch.int16).contiguous())
                done += n
        for seq in range(nb):
            B.cas_kv_set_len(self.kv, seq, self.ctx_len)
        torch.cuda.synchronize()
        mats = [L[n] for L in layers for n in dims] + [head]
        self.draft_w = sum(m.desc.rows * (m.desc.bw + m.desc.sw) * 4 for m in mats)
        self.verify_w = sum(m.desc.rows * (m.desc.bw + m.desc.sw + m.desc.lw + m.desc.pw) * 4 for m in mats)
        d = self.kv.desc
        bmw = 5 if kv_mx else 4   # bitmap words (+ one word of block exponents) per cached vector
        per_tok_draft = 2 * shape.n_layers * shape.n_kv_heads * 4 * (bmw + d.sw)
        per_tok_full = 2 * shape.n_layers * shape.n_kv_heads * 4 * (bmw + d.sw + d.lw + d.pw)
        self.draft_kv = per_tok_draft * self.ctx_len
        self.verify_kv = per_tok_full * self.ctx_len
        self.values = sum(m.desc.rows * m.desc.cols for m in mats)
        # a pass reads the weights once for all sequences and every sequence's cache; the
        # verification columns go into passes of at most 32 columns
        per_pass = max(1, min(nb, 32 // (self.k + 1)))
        self.draft_kv *= nb
        self.verify_kv *= nb
        self.verify_w *= (nb + per_pass - 1) // per_pass
        self.bytes_per_step = self.k * (self.draft_w + self.draft_kv) + self.verify_w + self.verify_kv
        self.pending = [1] * nb
        self.accepted, self.rounds = 0, 0
        self.config = {"workload": f"{name}-shaped random-init model ({shape.n_layers} layers, vocab {shape.vocab}, "
                                   f"{self.values / 1e9:.2f} G encoded weights), batch {nb}, KV context {self.ctx_len} "
                                   f"(synthetic K/V, 4 outlier key channels per head), draft length k={self.k}, "
                                   "greedy acceptance; weights + KV in Cassandra format",
                       "keep_permille": args.keep, "trunc_bits": args.trunc, "k": self.k, "context": self.ctx_len,
                       "kv_exp_mode": "shared" if kv_mx else "raw",
                       "step": "one speculative round: k draft passes + verify(k+1) + accept + commit"}

    def step(self):
        B, nb = self.B, self.batch
        if nb == 1:
            res = [B.cas_spec_round(self.ctx, self.model, self.kv, 0, self.pending[0], self.k)]
        else:
            res = B.cas_spec_round_multi(self.ctx, self.model, self.kv, list(range(nb)), self.pending, self.k)
        for seq, (n, out) in enumerate(res):
            self.pending[seq] = out[-1]
            self.accepted += n
            # keep the context length fixed across steps (roll the committed tokens back)
            B.cas_kv_set_len(self.kv, seq, self.ctx_len)
        self.rounds += 1

    def _chain_buffers(self):
        torch, shape = self.torch, self.shape
        gen = torch.Generator(device="cuda")
        gen.manual_seed(4321)
        # seeded N(0,1) activations (the residual stream h is updated in place by the chain)
        z = lambda n, c=1: torch.randn((c, n), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
        nb, nv = self.batch, min(16, self.batch * (self.k + 1))
        return {"h": z(shape.hidden, nb), "ao": z(shape.q_dim, nb), "act": z(shape.ffn, nb),
                "y": torch.empty((nv, max(shape.vocab, 2 * shape.ffn)), dtype=torch.float32, device="cuda"),
                "X": {c: z(c, nv) for c in (shape.hidden, shape.q_dim, shape.ffn)}}

    def _draft_gemv_chain(self, buf):
        """The draft-GEMV launches of one draft pass, back to back, with the same fused
        variants and shapes as in the model step."""
        B, ctx, eps = self.B, self.ctx, self.shape.rms_eps
        h, ao, act, y = buf["h"], buf["ao"], buf["act"], buf["y"]
        for L in self.layers:
            B.cas_gemv_draft_fused(ctx, L["wqkv"], h, y=y[:self.batch], gain=L["g_attn"], eps=eps, epilogue=0)
            B.cas_gemv_draft_fused(ctx, L["wo"], ao, epilogue=1, out16=h)
            B.cas_gemv_draft_fused(ctx, L["wgu"], h, gain=L["g_ffn"], eps=eps, epilogue=2, out16=act)
            B.cas_gemv_draft_fused(ctx, L["wd"], act, epilogue=1, out16=h)
        B.cas_gemv_draft_fused(ctx, self.head, h, y=y[:self.batch], gain=self.g_final, eps=eps, epilogue=0)

    def _verify_gemm_chain(self, buf):
        B, ctx, X, y = self.B, self.ctx, buf["X"], buf["y"]
        for L in self.layers:
            for n in ("wqkv", "wo", "wgu", "wd"):
                B.cas_gemm_verify(ctx, L[n], X[L[n].desc.cols], y[:, : L[n].desc.rows])
        B.cas_gemm_verify(ctx, self.head, X[self.head.desc.cols], y[:, : self.head.desc.rows])

    def _time_chain(self, fn, buf, reps=3):
        torch = self.torch
        fn(buf)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()                      # events on the stream the kernels are launched on
        for _ in range(reps):
            fn(buf)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    def roofline_pass(self):
        """Dominant kernel = fused draft decode+GEMV.  Its launches of one draft pass are replayed
        back to back between two HIP events (bracketing every launch of the interleaved model
        step with events would add the event overhead to each of them); the other streaming
        kernels are reported from per-launch event brackets inside two model steps."""
        B, ctx = self.B, self.ctx
        buf = self._chain_buffers()
        n = 4 * len(self.layers) + 1
        td = self._time_chain(self._draft_gemv_chain, buf)
        tv = self._time_chain(self._verify_gemm_chain, buf)
        B.cas_prof_reset(ctx)
        B.cas_prof_enable(ctx, True)
        acc0, r0 = self.accepted, self.rounds
        for _ in range(2):
            self.step()
        B.cas_prof_enable(ctx, False)
        self.accepted, self.rounds = acc0, r0
        self.prof = {name: B.cas_prof_read(ctx, cls) for name, cls in (("attn_draft", 2), ("attn_verify", 3))}
        B.cas_prof_reset(ctx)
        self.prof["gemv_draft"] = (n, td * 1e3, self.draft_w)
        self.prof["gemm_verify"] = (n, tv * 1e3, self.verify_w)
        ach = self.draft_w / td / 1e9
        # HBM-side bytes per launch from hardware counters (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on
        # `bench.py --workload probe-linear`; FETCH_SIZE scaled by 2.000, WRITE_SIZE by 1.000 after
        # calibration with a plain copy of known size): fetch / algorithmic bytes of the draft GEMV
        # measured per matrix shape of the 8B model, 1.035 for any other shape (the weighted mean);
        # every 4-byte output is written as a 32-byte sector (neighbouring rows belong to workgroups
        # on different XCDs).
        ratio = {(6144, 4096): 1.040, (4096, 4096): 1.044, (28672, 4096): 1.037, (4096, 14336): 1.027,
                 (128256, 4096): 1.030}
        mats = [L[n] for L in self.layers for n in ("wqkv", "wo", "wgu", "wd")] + [self.head]
        fetch = sum(ratio.get((m.desc.rows, m.desc.cols), 1.035) * m.desc.rows * (m.desc.bw + m.desc.sw) * 4
                    for m in mats)
        traffic = (fetch + 32.0 * sum(m.desc.rows for m in mats)) / n
        return {"bound": "hbm", "kernel": "gemv_draft_kernel", "achieved": ach, "peak": 8000.0, "unit": "GB/s",
                "frac": ach / 8000.0, "traffic": traffic, "launches": n, "avg_launch_us": td / n * 1e6,
                "bytes_per_launch": self.draft_w / n,
                "traffic_source": "profiles/pmc_gemv_draft_gemm_verify_llama3_8b_shapes.md (fetch / algorithmic "
                                  "ratio measured per matrix shape, applied to this run's launches; shapes "
                                  "outside that table use the weighted mean 1.035 and are an extrapolation)"}

    def _time_passes(self, reps=3):
        """Wall time of one draft pass, one verification pass (k+1 columns) and one plain decode
        step (verification with a single column) of the whole model, by HIP events."""
        torch, B, ctx = self.torch, self.B, self.ctx
        nb, k = self.batch, self.k
        seqs = list(range(nb))
        tok = torch.ones(nb * (k + 1), dtype=torch.int32, device="cuda")
        out = torch.empty(nb * (k + 1), dtype=torch.int32, device="cuda")

        def timed(fn, reps=reps):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        t_draft = timed(lambda: B.cas_draft_step_multi(ctx, self.model, self.kv, seqs, [0] * nb, tok[:nb], out[:nb]))
        t_verify = timed(lambda: B.cas_verify_step_multi(ctx, self.model, self.kv, seqs, [k] * nb, tok, out))
        t_plain = timed(lambda: B.cas_verify_step_multi(ctx, self.model, self.kv, seqs, [0] * nb, tok[:nb], out[:nb]))
        return t_draft, t_verify, t_plain

    def _forced_rounds(self, alpha, rounds=48, seed=11):
        """Tokens/s of whole rounds (k draft passes, verification, read-back of the targets,
        commit with the online KV encoder) when the number of accepted drafts is FORCED by a
        seeded Bernoulli(alpha) schedule instead of comparing tokens: synthetic acceptance,
        real work (the random-init model itself accepts nothing)."""
        import time
        import numpy as np
        torch, B, ctx, k, nb = self.torch, self.B, self.ctx, self.k, self.batch
        seqs = list(range(nb))
        rng = np.random.Generator(np.random.Philox(seed))
        tok = torch.ones(nb * (k + 1), dtype=torch.int32, device="cuda")
        out = torch.empty(nb * (k + 1), dtype=torch.int32, device="cuda")

        def one_round():
            for i in range(k):
                B.cas_draft_step_multi(ctx, self.model, self.kv, seqs, [i] * nb, tok[:nb], out[:nb])
            B.cas_verify_step_multi(ctx, self.model, self.kv, seqs, [k] * nb, tok, out)
            out.cpu()                                   # the host needs the target tokens to accept
            emitted = 0
            for seq in seqs:
                draws = rng.random(k) < alpha
                n = k if draws.all() else int(np.argmin(draws))
                B.cas_commit(ctx, self.model, self.kv, seq, n)
                emitted += n + 1
            return emitted

        def reset():
            for seq in seqs:
                B.cas_kv_set_len(self.kv, seq, self.ctx_len)

        one_round()
        reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tokens = sum(one_round() for _ in range(rounds))
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        reset()
        return {"tokens_per_s": tokens / dt, "tokens_per_round": tokens / rounds, "rounds": rounds}

    def extra(self, ms_per_step):
        t_draft, t_verify, t_plain = self._time_passes()
        k = self.k
        # context: the same linear layers as plain bf16 through the vendor GEMV (torch.mv), one pass
        t_bf16 = t_own = None
        if self.dense:
            torch = self.torch
            xs = {c: torch.randn(c, device="cuda").to(torch.bfloat16) for c in {w.shape[1] for w in self.dense}}

            def chain():
                for w in self.dense:
                    torch.mv(w, xs[w.shape[1]])
            chain()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                chain()
            e1.record()
            torch.cuda.synchronize()
            t_bf16 = e0.elapsed_time(e1) / 3
            # and through the library's own dense kernel (cas_gemv_bf16)
            B = self.B
            ys = {r: torch.empty(r, device="cuda") for r in {w.shape[0] for w in self.dense}}
            xb = {c: v.view(torch.int16) for c, v in xs.items()}
            wd = [w.view(torch.int16) for w in self.dense]

            def own():
                for w in wd:
                    B.cas_gemv_bf16(self.ctx, w, xb[w.shape[1]], ys[w.shape[0]])
            own()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(3):
                own()
            e1.record()
            torch.cuda.synchronize()
            t_own = e0.elapsed_time(e1) / 3
        # the whole plain bf16 decode step (dense GEMVs, attention over an uncompressed bf16 cache of the
        # same context, norms and residuals as separate small kernels): the BFloat16 baseline
        t_dense_step = None
        if self.dense and self.batch == 1:
            torch, B, shape = self.torch, self.B, self.shape
            nl = shape.n_layers
            dl = [{n: self.dense[4 * l + i].view(torch.int16) for i, n in enumerate(("wqkv", "wo", "wgu", "wd"))}
                  for l in range(nl)]
            head = self.dense[4 * nl].view(torch.int16)
            kvd = shape.n_kv_heads * shape.head_dim
            max_pos = self.ctx_len + 1024
            gen = torch.Generator(device="cuda")
            gen.manual_seed(99)
            kc = torch.randn((nl, max_pos, kvd), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
            vc = torch.randn((nl, max_pos, kvd), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
            tin = torch.ones(1, dtype=torch.int32, device="cuda")
            tout = torch.empty(1, dtype=torch.int32, device="cuda")
            step = lambda: B.cas_dense_decode_step(self.ctx, self.model, dl, head, kc, vc, self.ctx_len, tin, tout)
            step()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                step()
            e1.record()
            torch.cuda.synchronize()
            t_dense_step = e0.elapsed_time(e1) / 3
            del kc, vc
        # Speed model of Sec. 2.2: a round costs k t_draft + t_verify and yields accepted + 1 tokens.
        # The acceptance of a random-init model is ~0, so the table below uses an ASSUMED per-token
        # acceptance probability alpha (synthetic; the paper's acceptance table did not survive).
        synth_tps = {}
        for alpha in (0.0, 0.6, 0.8, 0.9, 1.0):
            exp_n = float(k) if alpha == 1.0 else sum(alpha ** i for i in range(1, k + 1))
            synth_tps[f"alpha={alpha}"] = self.batch * (exp_n + 1.0) / ((k * t_draft + t_verify) * 1e-3)
        out = {"tokens_per_s": (self.accepted + self.rounds * self.batch) / max(self.rounds, 1) / (ms_per_step * 1e-3),
               "accepted_per_round": self.accepted / max(self.rounds, 1),
               "draft_pass_ms": t_draft, "verify_pass_ms": t_verify, "plain_decode_step_ms": t_plain,
               "draft_pass_GBps": (self.draft_w + self.draft_kv) / (t_draft * 1e-3) / 1e9,
               "verify_pass_GBps": (self.verify_w + self.verify_kv) / (t_verify * 1e-3) / 1e9,
               "plain_decode_tokens_per_s": self.batch * 1e3 / t_plain,
               "context_vendor_bf16_gemv_pass_ms": t_bf16,
               "context_vendor_bf16_gemv_GBps": None if t_bf16 is None else 2.0 * self.values / (t_bf16 * 1e-3) / 1e9,
               "context_own_bf16_gemv_pass_ms": t_own,
               "context_own_bf16_gemv_GBps": None if t_own is None else 2.0 * self.values / (t_own * 1e-3) / 1e9,
               "context_own_bf16_decode_step_ms": t_dense_step,
               "context_own_bf16_decode_tokens_per_s": None if t_dense_step is None else 1e3 / t_dense_step,
               "tokens_per_s_at_assumed_acceptance": synth_tps,
               "tokens_per_s_forced_acceptance_schedule": {f"alpha={a}": self._forced_rounds(a)
                                                           for a in (0.0, 0.6, 0.8, 1.0)},
               "kernels": {}}
        for name, (n, ms, by) in self.prof.items():
            if n:
                out["kernels"][name] = {"launches": n, "avg_us": ms / n * 1e3, "GBps": by / (ms * 1e-3) / 1e9,
                                        "frac_of_peak": by / (ms * 1e-3) / 1e9 / 8000.0}
        return out


def run_probe(B, args):
    """Short fixed launch sequences for hardware-counter and kernel-trace runs (`bench.py --workload
    probe-linear | probe-attn`).  Each starts with three device-to-device copies of 256 MiB, the
    calibration kernel of known size for the FETCH_SIZE / WRITE_SIZE counters, and prints the
    algorithmic bytes of every launch that follows so that counter readings can be compared.

    probe-linear: draft GEMV (1 column) and verify GEMM (k+1 columns) on four distinct matrices of
    each 8B layer shape and one output head, then the unary-coded and shared-exponent draft GEMVs and
    verification GEMMs on the 28672 x 4096 matrices.  probe-attn: draft (1 column) and verification (k+1 columns) attention
    of one layer over a compressed cache of `--context` positions, six distinct layers."""
    import torch
    ctx = B.Context(workspace=torch.empty(256 << 20, dtype=torch.uint8, device="cuda"))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    k, keep, t = args.k, args.keep, args.trunc
    bf = lambda *s: torch.randn(s, device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
    src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()   # 256 MiB
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    print("copy_bytes_read", src.numel() * 4, "copy_bytes_written", src.numel() * 4)
    if args.workload == "probe-linear":
        shapes = (("wqkv", 6144, 4096, 4), ("wo", 4096, 4096, 4), ("wgu", 28672, 4096, 4), ("wd", 4096, 14336, 4),
                  ("head", 128256, 4096, 1))
        y = torch.empty((k + 1, 128256), device="cuda")
        for name, rows, cols, n in shapes:
            mats = [B.cas_encode_weight(ctx, _random_weight(torch, rows, cols, gen), keep, t) for _ in range(n)]
            x = bf(k + 1, cols)
            x1 = x[:1].contiguous()
            for _ in range(3):
                for m in mats:
                    B.cas_gemv_draft(ctx, m, x1, y[:1, :rows])
            for _ in range(3):
                for m in mats:
                    B.cas_gemm_verify(ctx, m, x, y[:, :rows])
            d = mats[0].desc
            print(f"{name} {rows}x{cols}: gemv_draft_algorithmic_bytes", rows * (d.bw + d.sw) * 4,
                  "gemm_verify_algorithmic_bytes", rows * (d.bw + d.sw + d.lw + d.pw) * 4, flush=True)
            if name == "wgu":
                yu = torch.empty(rows, device="cuda")
                umats = [B.cas_unary_encode(ctx, m) for m in mats]
                for _ in range(3):
                    for u in umats:
                        B.cas_gemv_draft_unary(ctx, u, x1, yu)
                xmats = [B.cas_mx_encode(ctx, m) for m in mats]
                for _ in range(3):
                    for xm in xmats:
                        B.cas_gemv_draft_mx(ctx, xm, x1, yu)
                for _ in range(3):
                    for xm in xmats:
                        B.cas_gemm_verify_mx(ctx, xm, x, y[:, :rows])
                for _ in range(3):
                    for u in umats:
                        B.cas_gemm_verify_unary(ctx, u, x, y[:, :rows])
                u, xd = umats[0].desc, xmats[0].desc
                print("gemv_draft_unary_algorithmic_bytes", rows * (d.bw + u.smw) * 4 + (u.ue_words + rows + 1) * 4)
                print("gemv_draft_mx_algorithmic_bytes", rows * (d.bw * 4 + d.bw + xd.fw * 4))
                print("gemm_verify_mx_algorithmic_bytes", rows * (d.bw * 4 + d.bw + (xd.fw + d.lw + d.pw) * 4))
                print("gemm_verify_unary_algorithmic_bytes (unary_expand_kernel, then gemm_verify_kernel on the "
                      "re-coded block)", rows * (d.bw + u.smw + d.lw + d.pw) * 4 + (u.ue_words + rows + 1) * 4,
                      flush=True)
                del umats, xmats
            del mats
    else:
        nq, nkv, ctx_len, layers = 32, 8, args.context, 6
        pages = (ctx_len + 64 + 63) // 64
        kv = B.KVCache(ctx, layers, nkv, n_pages=pages, max_seqs=1, max_pages_per_seq=pages, keep_permille=keep,
                       trunc_bits=t)
        for layer in range(layers):
            K = torch.randn((ctx_len, nkv, 128), device="cuda", generator=gen)
            K[:, :, torch.tensor([3, 40, 77, 100])] *= 10.0
            V = torch.randn((ctx_len, nkv, 128), device="cuda", generator=gen)
            B.cas_kv_set_len(kv, 0, 0)
            B.cas_kv_append(ctx, kv, layer, 0, K.to(torch.bfloat16).view(torch.int16).contiguous(),
                            V.to(torch.bfloat16).view(torch.int16).contiguous())
        B.cas_kv_set_len(kv, 0, ctx_len)
        Q, Kn, Vn = bf(k + 1, nq, 128), bf(k + 1, nkv, 128), bf(k + 1, nkv, 128)
        for _ in range(2):
            for layer in range(layers):
                B.cas_attention(ctx, kv, layer, 0, False, Q[:1].contiguous(), Kn[:1].contiguous(), Vn[:1].contiguous())
        for _ in range(2):
            for layer in range(layers):
                B.cas_attention(ctx, kv, layer, 0, True, Q, Kn, Vn)
        d = kv.desc
        print("attn_draft_algorithmic_bytes", 2 * nkv * 4 * (4 + d.sw) * ctx_len)
        print("attn_verify_algorithmic_bytes", 2 * nkv * 4 * (4 + d.sw + d.lw + d.pw) * ctx_len, flush=True)
    torch.cuda.synchronize()


def measure_format_grid(B, args, dev, keeps, truncs, layer_counts=(2, 8), reps=6):
    """Measured cost of every format of a grid (Sec. 7.2.2 searches such a grid; its Eq. 2 prices a
    format by the bits the draft reads, this prices it by time on this machine): for every
    (keep_permille, trunc_bits) pair, weights and cache of a model of the benchmark's shape are
    encoded with layer_counts[0] and layer_counts[1] decoder layers (plus embedding and output
    head), one draft pass, one verification pass of k + 1 columns and one plain decode step are
    timed by HIP events at the benchmark's context, and the times are extended linearly in the
    number of layers to args.layers.  Returns {"t_draft": [[s]], "t_verify": [[s]], "t_plain": [[s]]}."""
    import copy
    import torch
    full = args.layers
    l0, l1 = layer_counts
    out = {"t_draft": [], "t_verify": [], "t_plain": []}
    for kp in keeps:
        rows = {n: [] for n in out}
        for t in truncs:
            times = []
            for nl in (l0, l1):
                a = copy.copy(args)
                a.keep, a.trunc, a.layers = kp, t, nl
                wl = ModelRoundWorkload(B, a, dev)
                times.append(wl._time_passes(reps))      # ms: draft, verify, plain
                del wl
                torch.cuda.empty_cache()
            for i, n in enumerate(("t_draft", "t_verify", "t_plain")):
                per_layer = (times[1][i] - times[0][i]) / (l1 - l0)
                rows[n].append((times[0][i] + per_layer * (full - l0)) * 1e-3)
        for n in out:
            out[n].append(rows[n])
    return out


def run_tune(B, args, dev):
    """`bench.py --workload tune`: the format search driven by measured pass times.  The acceptance
    rate of every grid point is the user's (one number for all points with --alpha, or a JSON file
    with a [n_keep][n_trunc] table with --alpha-grid): it needs a trained model and a development
    set, which this build does not have.  Prints one JSON object: the measured times, tokens/s of
    every point under the speed model, Eq. 2's J for comparison and the two picks."""
    import json
    keeps = [int(x) for x in args.tune_keeps.split(",")]
    truncs = [int(x) for x in args.tune_truncs.split(",")]
    if args.alpha_grid:
        alpha = json.load(open(args.alpha_grid))
    else:
        alpha = [[args.alpha for _ in truncs] for _ in keeps]
    m = measure_format_grid(B, args, dev, keeps, truncs)
    best, rates = B.cas_tune_measured(alpha, m["t_draft"], m["t_verify"], args.k)
    if args.model == "70b":
        hid, nl, nq, nkv, ffn = 8192, args.layers, 64, 8, 28672
    else:
        hid, nl, nq, nkv, ffn = 4096, args.layers, 32, 8, 14336
    shape_w = nl * ((nq + 2 * nkv) * 128 * hid + hid * nq * 128 + 2 * ffn * hid + hid * ffn) + 128256 * hid
    s_kv = 2.0 * nl * nkv * 128 * args.context
    j = [[B.cas_objective(alpha[i][jj], float(shape_w), keeps[i], truncs[jj], s_kv, keeps[i], truncs[jj])
          for jj in range(len(truncs))] for i in range(len(keeps))]
    bj = B.cas_tune_grid(alpha, keeps, truncs, float(shape_w), s_kv, args.keep, args.trunc)
    speedup = [[B.cas_speed_model(alpha[i][jj], args.k, m["t_draft"][i][jj], m["t_verify"][i][jj],
                                  m["t_plain"][i][jj])[2] for jj in range(len(truncs))] for i in range(len(keeps))]
    print(json.dumps({"workload": "format search on measured pass times", "k": args.k, "context": args.context,
                      "keep_permille": keeps, "trunc_bits": truncs, "alpha": alpha, "alpha_source": "user-supplied",
                      "t_draft_s": m["t_draft"], "t_verify_s": m["t_verify"], "t_plain_s": m["t_plain"],
                      "tokens_per_s": rates, "speedup_over_plain_decode_from_the_same_format": speedup,
                      "best_by_measured_time": {"keep_permille": keeps[best[0]], "trunc_bits": truncs[best[1]]},
                      "eq2_J": j, "best_by_eq2_bits": {"keep_permille": keeps[bj[0]], "trunc_bits": truncs[bj[1]]}}))


def run_exp_modes(B, args, dev):
    """`bench.py --workload exp-modes`: pass times of the whole model with the speculation data of
    every linear layer in the raw, the unary-coded and the shared-exponent form (Sec. 4.2), on the
    same weights, cache and context.  Context figures, one JSON object; the metric's workload is
    the raw form."""
    import json
    import torch
    wl = ModelRoundWorkload(B, args, dev)
    ctx, model = wl.ctx, wl.model
    names = ("wqkv", "wo", "wgu", "wd")
    mats = [(l, w, L[n]) for l, L in enumerate(wl.layers) for w, n in enumerate(names)] + [(-1, 0, wl.head)]
    kv_d, kv_v = wl.draft_kv, wl.verify_kv

    def report(draft_bytes, verify_bytes):
        td, tv, tp = wl._time_passes(reps=3)
        return {"draft_pass_ms": td, "verify_pass_ms": tv, "plain_step_ms": tp,
                "draft_pass_bytes": draft_bytes + kv_d, "verify_pass_bytes": verify_bytes + kv_v,
                "draft_pass_GBps": (draft_bytes + kv_d) / td / 1e6, "verify_pass_GBps": (verify_bytes + kv_v) / tv / 1e6,
                "bits_per_value_draft": 8.0 * draft_bytes / wl.values, "bits_per_value_verify": 8.0 * verify_bytes / wl.values}

    out = {"workload": wl.config["workload"], "k": wl.k, "context": wl.ctx_len,
           "keep_permille": args.keep, "trunc_bits": args.trunc, "kv_exp_mode": wl.config["kv_exp_mode"],
           "kv_bytes_draft_pass": kv_d, "kv_bytes_verify_pass": kv_v}
    out["raw"] = report(wl.draft_w, wl.verify_w)
    # unary-coded exponents: lossless, verification gives the raw form's bits
    d_b = v_b = 0
    for l, w, m in mats:
        uw = B.cas_unary_encode(ctx, m)
        model.use_unary(l, w, uw)
        u, d = uw.desc, uw.desc.base
        b = d.rows * (d.bw + u.smw) * 4 + u.ue_words * 4 + (d.rows + 1) * 4 + 512
        d_b += b
        v_b += b + d.rows * (d.lw + d.pw) * 4
    torch.cuda.synchronize()
    out["unary"] = report(d_b, v_b)
    for l, w, m in mats:
        model.use_unary(l, w, None)
    model._unary = {}
    # shared exponents: the converted matrices are the weights
    d_b = v_b = 0
    for l, w, m in mats:
        mw = B.cas_mx_encode(ctx, m)
        model.use_mx(l, w, mw)
        x, d = mw.desc, mw.desc.base
        b = d.rows * (d.bw * 4 + x.ew + x.fw * 4)
        d_b += b
        v_b += b + d.rows * (d.lw + d.pw) * 4
    torch.cuda.synchronize()
    out["mx"] = report(d_b, v_b)
    print(json.dumps(out))


def build(B, args, dev):
    if args.workload == "linear":
        return LinearRoundWorkload(B, args, dev)
    return ModelRoundWorkload(B, args, dev)
