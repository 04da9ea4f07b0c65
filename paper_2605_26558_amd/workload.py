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


def build(B, args, dev):
    return LinearRoundWorkload(B, args, dev)
