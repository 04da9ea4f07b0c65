#!/usr/bin/env python3
"""Writes tests/golden/llama70b_layer_logits.txt: the oracle's logits of the verification pass
(k + 1 = 9 columns) and of the first draft pass for the Llama-3-70B-shaped one-layer case of
synth.llama70b_layer_case (Sec. 4.1 target and draft inference; Sec. 2.2 batched verification).

Calls only synth (inputs) and oracle/ (arithmetic).  The 0.86 G weights go through the oracle's
own encode -> decode in chunks of rows (rows are independent selection groups, Sec. 4.2), which
takes some ten minutes on 8 cores; the GPU test then only has to read the stored logits.

    python tests/golden/make_llama70b_layer_logits.py
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth                                        # noqa: E402
from oracle import cassandra_oracle as O            # noqa: E402

OUT = os.path.join(ROOT, "tests", "golden", "llama70b_layer_logits.txt")


def u16(t):
    return t.numpy().view(np.uint16)


def decoded_views(w, act, keep, t, chunk=2048):
    """(draft view, full view) of a matrix as float64, through encode_weight / decode_*."""
    rows, cols = w.shape
    wd = np.empty((rows, cols), dtype=np.float64)
    wf = np.empty((rows, cols), dtype=np.float64)
    for r0 in range(0, rows, chunk):
        p = O.encode_weight(w[r0:r0 + chunk], keep, t, act)
        wd[r0:r0 + chunk] = O.bf16_to_f64(O.decode_draft(p))
        full = O.decode_full(p)
        assert np.array_equal(full, w[r0:r0 + chunk])
        wf[r0:r0 + chunk] = O.bf16_to_f64(full)
    return wd, wf


def main():
    case = synth.llama70b_layer_case("cpu")
    shape, keep, t, k, L = case["shape"], case["keep"], case["t"], case["k"], case["ctx_len"]
    tab = synth.rope_table(L + 64, shape.head_dim, shape.rope_theta)
    om = O.OracleModel.__new__(O.OracleModel)       # weights are injected below, chunk by chunk
    om.s, om.rope_tab, om.kv_keep, om.kv_t = shape, tab, keep, t
    om.embed = u16(case["embed"]())
    om.g_final = u16(case["gain"](2))
    om.layers = [{"g_attn": u16(case["gain"](0)), "g_ffn": u16(case["gain"](1))}]
    om._dec = {}
    t0 = time.time()
    for name in ("wqkv", "wo", "wgu", "wd", "lm_head"):
        wd, wf = decoded_views(u16(case["weight"](name)), case["act_norm"](name).numpy(), keep, t)
        key = None if name == "lm_head" else 0
        om._dec[(key, name, True)], om._dec[(key, name, False)] = wd, wf
        print(f"{name} decoded, {time.time() - t0:.0f} s", flush=True)
    K, V = u16(case["K"]()), u16(case["V"]())
    pk, pv = O.encode_kv(K.reshape(-1, 128), keep, t), O.encode_kv(V.reshape(-1, 128), keep, t)
    views = {True: (O.decode_draft(pk).reshape(K.shape), O.decode_draft(pv).reshape(V.shape)),
             False: (O.decode_full(pk).reshape(K.shape), O.decode_full(pv).reshape(V.shape))}
    assert np.array_equal(views[False][0], K) and np.array_equal(views[False][1], V)
    om._cache_kv = lambda layer_index, draft: views[draft]
    om.cache_len = lambda: L
    tokens = case["tokens"]
    verify, _ = om.forward(tokens, draft=False)
    empty = [(np.zeros((0, shape.n_kv_heads, 128), np.uint16),) * 2]
    draft, _ = om.forward(tokens[:1], draft=True, extra_kv=empty)
    gnorm = np.linalg.norm(O.bf16_to_f64(om.g_final))
    rows = {"verify_row_norm_times_gain_norm": np.linalg.norm(om._dec[(None, "lm_head", False)], axis=1) * gnorm,
            "draft_row_norm_times_gain_norm": np.linalg.norm(om._dec[(None, "lm_head", True)], axis=1) * gnorm}
    with open(OUT, "w") as f:
        f.write("# Written by tests/golden/make_llama70b_layer_logits.py (oracle only); inputs: synth.llama70b_layer_case.\n")
        f.write("# Logits of the verification pass over 9 columns and of the first draft pass (Sec. 4.1), float64;\n")
        f.write("# *_row_norm_times_gain_norm = |W_row| |g_final| of the view the pass reads (scale of the tolerance).\n")
        for c in range(k + 1):
            f.write(f"verify_logits_col{c} " + " ".join(f"{v:.17g}" for v in verify[c]) + "\n")
        f.write("draft_logits_col0 " + " ".join(f"{v:.17g}" for v in draft[0]) + "\n")
        for name, v in rows.items():
            f.write(name + " " + " ".join(f"{x:.17g}" for x in v) + "\n")
    print("wrote", OUT, f"{time.time() - t0:.0f} s")


if __name__ == "__main__":
    main()
