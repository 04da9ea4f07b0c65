"""Small driver for hardware-counter runs on the attention kernels: one device-to-device copy of
known size (calibration), then draft (1 column) and verification (7 columns) attention of one
layer over a compressed cache of 8192 committed positions (8 kv heads, 32 query heads, paper-
default format), several distinct layers so the cache is not re-read from L2.  Prints the
algorithmic bytes of a call so counter readings can be compared."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    import torch
    from paper_2605_26558_amd import binding as B
    ctx = B.Context(workspace=torch.empty(64 << 20, dtype=torch.uint8, device="cuda"))
    nq, nkv, ctx_len, layers, k = 32, 8, 8192, 6, 6
    pages = (ctx_len + 64 + 63) // 64
    kv = B.KVCache(ctx, layers, nkv, n_pages=pages, max_seqs=1, max_pages_per_seq=pages)
    gen = torch.Generator(device="cuda"); gen.manual_seed(3)
    for layer in range(layers):
        K = torch.randn((ctx_len, nkv, 128), device="cuda", generator=gen)
        K[:, :, torch.tensor([3, 40, 77, 100])] *= 10.0
        V = torch.randn((ctx_len, nkv, 128), device="cuda", generator=gen)
        B.cas_kv_set_len(kv, 0, 0)
        B.cas_kv_append(ctx, kv, layer, 0, K.to(torch.bfloat16).view(torch.int16).contiguous(),
                        V.to(torch.bfloat16).view(torch.int16).contiguous())
    B.cas_kv_set_len(kv, 0, ctx_len)
    bf = lambda *s: torch.randn(s, device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
    Q, Kn, Vn = bf(k + 1, nq, 128), bf(k + 1, nkv, 128), bf(k + 1, nkv, 128)
    src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()   # 256 MiB
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)
    for _ in range(2):
        for layer in range(layers):
            B.cas_attention(ctx, kv, layer, 0, False, Q[:1].contiguous(), Kn[:1].contiguous(), Vn[:1].contiguous())
    for _ in range(2):
        for layer in range(layers):
            B.cas_attention(ctx, kv, layer, 0, True, Q, Kn, Vn)
    torch.cuda.synchronize()
    d = kv.desc
    per_tok_draft = 2 * nkv * 4 * (4 + d.sw)
    per_tok_full = 2 * nkv * 4 * (4 + d.sw + d.lw + d.pw)
    print("copy_bytes_read", src.numel() * 4)
    print("attn_draft_algorithmic_bytes", per_tok_draft * ctx_len)
    print("attn_verify_algorithmic_bytes", per_tok_full * ctx_len)


if __name__ == "__main__":
    main()
