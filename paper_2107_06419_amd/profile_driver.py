"""Workload driver for rocprofv3 runs:  rocprofv3 <options> -- python3 -m paper_2107_06419_amd.profile_driver ...

Launches, in this order and each `--reps` times on one workload: the fused kernel, optionally the
three unfused kernels, and a plain device-to-device copy of a known size (the calibration kernel
for byte counters such as FETCH_SIZE / WRITE_SIZE).
"""
import argparse
import sys


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg2_long_16k")
    ap.add_argument("--shape", default="", help="B,H,N,d,mask of a bf16 problem to run instead of a named workload")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--unfused", action="store_true")
    ap.add_argument("--copy-mib", type=int, default=1024, help="size of the calibration copy (MiB read + MiB written)")
    ap.add_argument("--cache", default="", help="H,Nq,Nk,d: instead of the above, a causal segment of Nq queries over Nk cached keys "
                                                "through flat_attn_fwd_cross and flat_attn_fwd_splitkv")
    ap.add_argument("--mix", action="store_true", help="instead of the above, the four levels of the instruction-mix probe")
    ap.add_argument("--mfma", default="", choices=["", "constant", "random"], help="instead of the above, the MFMA-only probe on these operands")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2107_06419_amd as fa
    from paper_2107_06419_amd import synth

    if args.mfma:
        sink = torch.empty(fa.flat_attn_mfma_probe_sink_bytes() // 4, dtype=torch.float32, device="cuda")
        for _ in range(args.reps):
            fa.flat_attn_mfma_probe(sink, 16000, args.mfma == "random")
        torch.cuda.synchronize()
        print("profile_driver done mfma", args.mfma, flush=True)
        return 0
    if args.mix:
        sink = torch.empty(fa.flat_attn_mix_probe_sink_bytes() // 4, dtype=torch.float32, device="cuda")
        src = torch.randn(fa.flat_attn_mix_probe_src_bytes() // 2, device="cuda").to(torch.bfloat16)
        for level in range(4):
            for _ in range(args.reps):
                fa.flat_attn_mix_probe(sink, src, level, 500)
            torch.cuda.synchronize()
        print("profile_driver done mix", flush=True)
        return 0
    if args.cache:
        H, Nq, Nk, d = (int(t) for t in args.cache.split(","))
        scale = float(np.float32(d ** -0.5))
        tq = torch.randn(1, H, Nq, d, device="cuda").to(torch.bfloat16)
        tk = torch.randn(1, H, Nk, d, device="cuda").to(torch.bfloat16)
        tv = torch.randn(1, H, Nk, d, device="cuda").to(torch.bfloat16)
        to = torch.empty_like(tq)
        ws = torch.empty(fa.flat_attn_fwd_splitkv_workspace_bytes(1, H, Nq, Nk, d, 0) // 4, dtype=torch.float32, device="cuda")
        for _ in range(args.reps):
            fa.flat_attn_fwd_cross(tq, tk, tv, to, scale, 1)
        torch.cuda.synchronize()
        for _ in range(args.reps):
            fa.flat_attn_fwd_splitkv(tq, tk, tv, to, scale, 1, None, 0, ws)
        torch.cuda.synchronize()
        if args.copy_mib > 0:  # the copy of known size that calibrates FETCH_SIZE / WRITE_SIZE
            n = args.copy_mib * (1 << 20) // 4
            src = torch.ones(n, dtype=torch.float32, device="cuda")
            dst = torch.empty_like(src)
            torch.cuda.synchronize()
            for _ in range(args.reps):
                dst.copy_(src)
            torch.cuda.synchronize()
        print("profile_driver done cache", args.cache, "splits", fa.flat_attn_fwd_splitkv_splits(1, H, Nq, Nk, d, 0), flush=True)
        return 0
    if args.shape:
        B, H, N, d, mask = (int(t) for t in args.shape.split(","))
        w = synth.custom("shape_" + args.shape.replace(",", "_"), B, H, N, d, "bf16", mask, seed=1)
    else:
        w = synth.WORKLOADS[args.workload]
    q, k, v = synth.make_qkv(w)

    def dev(x):
        return torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda().view(torch.bfloat16)

    dq, dk, dv = dev(q), dev(k), dev(v)
    out = torch.empty_like(dq)
    for _ in range(args.reps):
        fa.flat_attn_fwd(dq, dk, dv, out, w.scale, w.mask)
    torch.cuda.synchronize()
    if args.unfused:
        ws = torch.empty(fa.flat_attn_unfused_workspace_bytes(w.B, w.H, w.N, w.d) // 4, dtype=torch.float32, device="cuda")
        for _ in range(args.reps):
            fa.flat_attn_unfused(dq, dk, dv, out, w.scale, w.mask, ws)
        torch.cuda.synchronize()
        del ws
    if args.copy_mib > 0:
        n = args.copy_mib * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(args.reps):
            dst.copy_(src)
        torch.cuda.synchronize()
    print("profile_driver done", w.name, flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
