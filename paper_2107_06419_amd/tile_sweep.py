"""Measured tile-shape sweep of the fused bf16 kernel:  python -m paper_2107_06419_amd.tile_sweep [--small] [--out FILE]

The paper chooses tile sizes by exhaustive search over a cost model (section 6.1, map-space exploration)
and names the trade-off of the row granularity (section 5.3).  This tool does the search by timing: every
tile shape the library was built with (flat_attn_tile_shape_*) runs on a set of problem shapes through
flat_attn_fwd_tile, and the table of times is printed as Markdown.  Each shape's output is compared with
the default shape's (index 0) on the same input, so a row in the table is also a consistency check.
With --small it times launches of few row blocks instead (1 to 128 heads of 128 to 4096 positions), the 256-row
default shape against the 128-row shapes: the table the small-launch rule of flat_attn_fwd was read off.
Needs a GPU; inputs are the seeded synthetic tensors of paper_2107_06419_amd.synth.
"""
from __future__ import annotations

import argparse
import sys

# (label, B, H, N, d, mask)
PROBLEMS = [
    ("cfg1 encoder 4K", 8, 16, 4096, 64, 0),
    ("cfg2 long 16K", 1, 16, 16384, 64, 0),
    ("cfg4 extreme 64K", 1, 8, 65536, 64, 0),
    ("short 1K", 8, 16, 1024, 64, 0),
    ("causal 8K", 2, 8, 8192, 64, 1),
    ("causal 16K", 1, 16, 16384, 64, 1),
    ("cfg3 wide causal 8K", 2, 8, 8192, 128, 1),
    ("wide 8K", 2, 8, 8192, 128, 0),
    ("wide 16K", 1, 8, 16384, 128, 0),
    ("wide short 1K", 8, 16, 1024, 128, 0),
    ("wide causal 32K", 1, 4, 32768, 128, 1),
    ("narrow 16K", 1, 32, 16384, 32, 0),
    ("narrow causal 8K", 2, 16, 8192, 32, 1),
    ("d96 16K", 1, 12, 16384, 96, 0),
    ("d96 causal 8K", 2, 8, 8192, 96, 1),
    ("d256 16K", 1, 4, 16384, 256, 0),
    ("d256 causal 8K", 2, 4, 8192, 256, 1),
]


def time_launch(fn, flops: float, min_warm_ms: float = 40.0, reps: int = 30) -> float:
    """Average milliseconds per launch after the clocks have ramped (HIP events on the current stream)."""
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    fn()
    e1.record()
    torch.cuda.synchronize()
    once = max(e0.elapsed_time(e1), 1e-3)
    for _ in range(int(min_warm_ms / once) + 1):
        fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def small_launches(reps: int) -> str:
    """Median microseconds per launch of the default shape and the 128-row shapes on small problems."""
    import statistics

    import numpy as np
    import torch

    import paper_2107_06419_amd as fa
    from paper_2107_06419_amd import synth

    def dev(x):
        return torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda().view(torch.bfloat16)

    def median_us(fn):
        for _ in range(30):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        return statistics.median(a.elapsed_time(b) for a, b in ev) * 1e3

    lines = ["One batch entry, BH heads of N positions; median of %d launches by HIP events after 30 warm-up launches, in" % reps,
             "microseconds.  blocks = BH * ceil(N / 256), the workgroups of the default shape; the last column is the time of",
             "shape 0 over the best time, with the best shape.", ""]
    for d, shapes in ((64, (0, 5, 7)), (128, (0, 2)), (32, (0, 1)), (96, (0, 1))):
        for i in shapes:
            t = fa.flat_attn_tile_shape_get(d, i).as_dict()
            lines.append(f"d = {d} shape {i}: {t['rows_per_workgroup']} rows ({t['wavefronts']} wavefronts x {t['rows_per_wavefront']}), "
                         f"{t['lds_stages']} stages, {fa.flat_attn_tile_shape_occupancy(d, i)} workgroups per CU")
    lines.append("")
    for d, shapes in ((64, (0, 5, 7)), (128, (0, 2)), (32, (0, 1)), (96, (0, 1))):
        for mask in (0, 1):
            lines.append(f"### d = {d}, {'causal' if mask else 'no mask'}")
            lines.append("")
            lines.append("| N | BH | blocks | " + " | ".join(f"shape {i}" for i in shapes) + " | shape 0 / best |")
            lines.append("|" + "---|" * (4 + len(shapes)))
            for N in (128, 256, 512, 1024, 2048, 4096):
                for BH in (4, 12, 32, 64, 128):
                    if BH * N > 64 * 4096:
                        continue
                    w = synth.custom(f"small_{d}_{N}_{BH}", 1, BH, N, d, "bf16", mask, seed=977 + N + BH + d)
                    q, k, v = synth.make_qkv(w)
                    dq, dk, dv = dev(q), dev(k), dev(v)
                    out = torch.empty_like(dq)
                    ts = [median_us(lambda: fa.flat_attn_fwd_tile(dq, dk, dv, out, w.scale, mask, i)) for i in shapes]
                    best = min(range(len(ts)), key=lambda i: ts[i])
                    lines.append(f"| {N} | {BH} | {BH * ((N + 255) // 256)} | " + " | ".join(f"{t:.1f}" for t in ts) +
                                 f" | {ts[0] / ts[best]:.2f} (shape {shapes[best]}) |")
                    print(lines[-1], file=sys.stderr, flush=True)
            lines.append("")
    return "\n".join(lines)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="", help="also write the Markdown table to this file")
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--small", action="store_true", help="time small launches (default shape against the 128-row shapes) instead")
    args = ap.parse_args()
    if args.small:
        text = small_launches(max(args.reps, 40))
        print(text)
        if args.out:
            with open(args.out, "w") as f:
                f.write(text + "\n")
        return 0

    import numpy as np
    import torch

    import paper_2107_06419_amd as fa
    from paper_2107_06419_amd import synth

    def dev(x):
        return torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda().view(torch.bfloat16)

    lines = []
    for d in (64, 128, 32, 96, 256):
        n = fa.flat_attn_tile_shape_count(d)
        shapes = [fa.flat_attn_tile_shape_get(d, i).as_dict() for i in range(n)]
        occ = [fa.flat_attn_tile_shape_occupancy(d, i) for i in range(n)]
        lines.append(f"### d = {d}: tile shapes")
        lines.append("")
        lines.append("| index | rows/workgroup (Br) | keys/tile (Bc) | wavefronts | rows/wavefront | LDS stages | LDS bytes | workgroups/CU |")
        lines.append("|---|---|---|---|---|---|---|---|")
        for i, (t, o) in enumerate(zip(shapes, occ)):
            lines.append(f"| {i}{' (default)' if i == 0 else ''} | {t['rows_per_workgroup']} | {t['keys_per_tile']} | {t['wavefronts']} | "
                         f"{t['rows_per_wavefront']} | {t['lds_stages']} | {t['lds_bytes']} | {o} |")
        lines.append("")
        lines.append(f"### d = {d}: milliseconds per launch (useful TFLOP/s), best shape in bold")
        lines.append("")
        lines.append("| problem (B,H,N,mask) | " + " | ".join(f"shape {i}" for i in range(n)) + " | max abs diff vs shape 0 |")
        lines.append("|---|" + "---|" * (n + 1))
        for label, B, H, N, dd, mask in PROBLEMS:
            if dd != d:
                continue
            w = synth.custom(label.replace(" ", "_"), B, H, N, d, "bf16", mask, seed=4242 + N + d + mask)
            q, k, v = synth.make_qkv(w)
            dq, dk, dv = dev(q), dev(k), dev(v)
            del q, k, v
            flops = 4.0 * B * H * N * N * d * (0.5 * (N + 1) / N if mask else 1.0)
            ref = None
            cells, worst = [], 0.0
            times = []
            for i in range(n):
                out = torch.full_like(dq, float("nan"))
                ms = time_launch(lambda: fa.flat_attn_fwd_tile(dq, dk, dv, out, w.scale, w.mask, i), flops, reps=args.reps)
                torch.cuda.synchronize()
                if ref is None:
                    ref = out.float()
                diff = (out.float() - ref).abs().max().item()
                if not diff <= 2e-2:
                    raise SystemExit(f"shape {i} of d={d} disagrees with shape 0 on {label}: {diff}")
                worst = max(worst, diff)
                times.append(ms)
                print(f"d={d} {label} shape {i}: {ms:.4f} ms", file=sys.stderr, flush=True)
            best = min(range(n), key=lambda i: times[i])
            for i, ms in enumerate(times):
                cell = f"{ms:.3f} ({flops / ms / 1e9:.0f})"
                cells.append(f"**{cell}**" if i == best else cell)
            lines.append(f"| {label} ({B},{H},{N},{'causal' if mask else 'none'}) | " + " | ".join(cells) + f" | {worst:.1e} |")
            del dq, dk, dv, ref, out
        lines.append("")
    text = "\n".join(lines)
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
