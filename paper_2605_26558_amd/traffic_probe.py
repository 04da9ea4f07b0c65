"""Small driver for hardware-counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE): one plain
device-to-device copy of known size (the calibration kernel) followed by draft-GEMV,
verify-GEMM, unary and shared-exponent draft-GEMV launches on Llama-3-8B gate/up shaped matrices (28672 x 4096, paper-default
format).  Prints the algorithmic bytes of each launch so counter readings can be compared."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    import torch
    from paper_2605_26558_amd import binding as B
    from paper_2605_26558_amd.workload import _random_weight
    ctx = B.Context(workspace=torch.empty(8 << 20, dtype=torch.uint8, device="cuda"))
    gen = torch.Generator(device="cuda"); gen.manual_seed(7)
    rows, cols, k = 28672, 4096, 6
    mats = [B.cas_encode_weight(ctx, _random_weight(torch, rows, cols, gen), 600, 4) for _ in range(4)]
    x = torch.randn((k + 1, cols), device="cuda", generator=gen).to(torch.bfloat16).view(torch.int16)
    x1 = x[:1].contiguous()
    y = torch.empty((k + 1, rows), device="cuda")
    src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()   # 256 MiB
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(3):
        dst.copy_(src)                       # reads 256 MiB, writes 256 MiB
    for _ in range(3):
        for m in mats:
            B.cas_gemv_draft(ctx, m, x1, y[:1])
    for _ in range(3):
        for m in mats:
            B.cas_gemm_verify(ctx, m, x, y)
    umats = [B.cas_unary_encode(ctx, m) for m in mats]     # unary-coded exponents of the same matrices
    yu = torch.empty(rows, device="cuda")
    for _ in range(3):
        for u in umats:
            B.cas_gemv_draft_unary(ctx, u, x1, yu)
    xmats = [B.cas_mx_encode(ctx, m) for m in mats]        # shared-exponent form of the same matrices
    for _ in range(3):
        for xm in xmats:
            B.cas_gemv_draft_mx(ctx, xm, x1, yu)
    torch.cuda.synchronize()
    d = mats[0].desc
    print("copy_bytes_read", src.numel() * 4, "copy_bytes_written", src.numel() * 4)
    print("gemv_draft_algorithmic_bytes", rows * (d.bw + d.sw) * 4)
    print("gemm_verify_algorithmic_bytes", rows * (d.bw + d.sw + d.lw + d.pw) * 4)
    u = umats[0].desc
    print("gemv_draft_unary_algorithmic_bytes", rows * (d.bw + u.smw) * 4 + (u.ue_words + rows + 1) * 4)
    xd = xmats[0].desc
    print("gemv_draft_mx_algorithmic_bytes", rows * (d.bw * 4 + d.bw + xd.fw * 4))


if __name__ == "__main__":
    main()
