"""Block-sparse sweep of the fused bf16 kernel:  python -m paper_2107_06419_amd.sparse_sweep [--out FILE]

The paper prunes the Logit/Attend matrix randomly at 50 % and asks whether the pair stays memory-bound when
run operator by operator and what fusion changes (section 8.2, compute-time / memory-time ratio C/M).  This
tool runs flat_attn_fwd_blocksparse on seeded random block patterns (256 rows x 64 keys) of several densities
and prints, per density: the kernel time, the useful TFLOP/s (density x dense flops), and C/M for the fused
kernel (measured time against its algorithmic bytes at 8 TB/s) next to C/M of an operator-by-operator
execution of the same pruned matrix (MFMA peak time against 16 bytes per kept logit).  Needs a GPU.
"""
from __future__ import annotations

import argparse
import sys

PROBLEMS = [("cfg2 shape", 1, 16, 16384, 64), ("wide 16K", 1, 8, 16384, 128)]
DENSITIES = [1.0, 0.75, 0.5, 0.25, 0.1]
HBM_BPS = 8.0e12
MFMA_FLOPS = 2.5e15


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2107_06419_amd as fa
    from paper_2107_06419_amd import synth
    from paper_2107_06419_amd.tile_sweep import time_launch

    def dev(x):
        return torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda().view(torch.bfloat16)

    lines = ["| problem (B,H,N,d) | density | tiles listed | ms | useful TFLOP/s | fused C/M | operator-by-operator C/M |", "|---|---|---|---|---|---|---|"]
    for label, B, H, N, d in PROBLEMS:
        w = synth.custom(label.replace(" ", "_"), B, H, N, d, "bf16", 0, seed=99 + d)
        q, k, v = synth.make_qkv(w)
        dq, dk, dv = dev(q), dev(k), dev(v)
        out = torch.empty_like(dq)
        n_rb, n_kt = -(-N // fa.binding.FLAT_SPARSE_BLOCK_ROWS), -(-N // fa.binding.FLAT_SPARSE_BLOCK_KEYS)
        dense_ms = time_launch(lambda: fa.flat_attn_fwd(dq, dk, dv, out, w.scale, 0), 0.0)
        for rho in DENSITIES:
            offs, ids = synth.random_block_pattern(B * H * n_rb, n_kt, rho, seed=int(rho * 1000) + d)
            d_offs = torch.from_numpy(offs.astype(np.int32)).cuda()
            d_ids = torch.from_numpy(ids.astype(np.int32)).cuda()
            ms = time_launch(lambda: fa.flat_attn_fwd_blocksparse(dq, dk, dv, out, w.scale, d_offs, d_ids), 0.0)
            kept = ids.size / float(B * H * n_rb * n_kt)
            flops = 4.0 * B * H * N * N * d * kept
            fused_bytes = 4.0 * B * H * N * d * 2 + (offs.size + ids.size) * 4      # Q, K, V, O once, plus the lists
            fused_cm = (ms * 1e-3) / (fused_bytes / HBM_BPS)
            unfused_cm = (flops / MFMA_FLOPS) / ((16.0 * kept * B * H * N * N + 4.0 * B * H * N * d * 2) / HBM_BPS)
            lines.append(f"| {label} ({B},{H},{N},{d}) | {rho:.2f} | {ids.size} ({100 * kept:.1f} %) | {ms:.3f} | {flops / ms / 1e9:.0f} | "
                         f"{fused_cm:.0f} | {unfused_cm:.3f} |")
            print(lines[-1], file=sys.stderr, flush=True)
        lines.append(f"| {label} dense kernel (flat_attn_fwd) | 1.00 | — | {dense_ms:.3f} | {4.0 * B * H * N * N * d / dense_ms / 1e9:.0f} | | |")
    text = "\n".join(lines)
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
