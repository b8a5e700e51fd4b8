#!/usr/bin/env python3
"""Benchmark of the fused attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one call of flat_attn_fwd (the whole fused Logit-softmax-Attend path) on one synthetic
batch of the named workload, inputs resident in HBM.  Prints ONE JSON line: whole-job throughput
in TFLOP/s (4*B*H*N^2*d flops per step; for a causal workload the useful 2*B*H*N*(N+1)*d), the
MFMA roofline of the fused kernel measured with HIP events inside the timed region, the unfused
baseline's time and HBM bytes for comparison, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA peak
PEAK_F32_TFLOPS = 157.3    # published fp32 matrix/vector peak (the fp32 variant runs on fp32 MFMA)
METRIC = "fused attention TFLOP/s and % bf16 MFMA peak at N=16K,d=64; HBM bytes vs unfused"


def load_traffic(workload: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), if a summary is committed."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg2_long_16k")
    ap.add_argument("--unfused-steps", type=int, default=3, help="timed launches of the unfused baseline (0 = skip)")
    ap.add_argument("--mfma-probe-launches", type=int, default=24, help="launches of the MFMA-only probe per operand kind (0 = skip)")
    ap.add_argument("--cpu-rows-per-head", type=int, default=16384, help="oracle sample size (0 = skip the cpu_baseline leg)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only: the heads of a batch are independent, so more GPUs would each take a share of them with no exchange; use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2107_06419_amd as fa
    from paper_2107_06419_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    fa.load_library()  # raises if the HIP library is not built: there is no fallback path

    w = synth.WORKLOADS[args.workload]
    is_bf16 = w.dtype == "bf16"
    if not is_bf16:
        args.unfused_steps = 0  # the unfused baseline exists for bf16 only
    q, k, v = synth.make_qkv(w)

    def dev(x):
        if not is_bf16:
            return torch.from_numpy(np.ascontiguousarray(x)).cuda()
        return torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda().view(torch.bfloat16)

    dq, dk, dv = dev(q), dev(k), dev(v)
    out = torch.empty_like(dq)
    stream = torch.cuda.current_stream()

    fwd = fa.flat_attn_fwd if is_bf16 else fa.flat_attn_fwd_f32

    def step():
        fwd(dq, dk, dv, out, w.scale, w.mask, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        starts[i].record(stream)
        step()
        ends[i].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    per_launch = sorted(s.elapsed_time(e) for s, e in zip(starts, ends))
    kernel_ms = sum(per_launch) / args.steps
    flops = w.flops_useful
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    kernel_tflops = flops / (kernel_ms * 1e-3) / 1e12

    elem = 2 if is_bf16 else 4
    fused_alg_bytes = 4 * w.B * w.H * w.N * w.d * elem                 # Q, K, V read once, O written once
    unfused_alg_bytes = fused_alg_bytes + 16 * w.B * w.H * w.N * w.N   # fp32 L: write, read, write in place, read
    traffic = load_traffic(w.name)

    unfused = None
    if args.unfused_steps > 0:
        nbytes = fa.flat_attn_unfused_workspace_bytes(w.B, w.H, w.N, w.d)
        ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
        out_u = torch.empty_like(dq)
        fa.flat_attn_unfused(dq, dk, dv, out_u, w.scale, w.mask, ws, stream)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(args.unfused_steps):
            fa.flat_attn_unfused(dq, dk, dv, out_u, w.scale, w.mask, ws, stream)
        torch.cuda.synchronize()
        unfused_ms = (time.perf_counter() - t2) * 1e3 / args.unfused_steps
        unfused = {"ms_per_step": round(unfused_ms, 4), "tflops": round(flops / (unfused_ms * 1e-3) / 1e12, 2),
                   "algorithmic_hbm_bytes": unfused_alg_bytes,
                   "algorithmic_hbm_gbps": round(unfused_alg_bytes / (unfused_ms * 1e-3) / 1e9, 1),
                   "workspace_bytes": nbytes,
                   "max_abs_diff_vs_fused": float((out_u.float() - out.float()).abs().max().item())}
        del ws, out_u

    # what the matrix pipe sustains by itself on this GPU (clock under load depends on the operands' power draw)
    probe = None
    if args.mfma_probe_launches > 0:
        sink = torch.empty(fa.flat_attn_mfma_probe_sink_bytes() // 4, dtype=torch.float32, device="cuda")
        iters = 16000
        probe = {}
        for name, rnd in (("constant_operands_tflops", False), ("random_operands_tflops", True)):
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.mfma_probe_launches + 1)]
            evs[0].record(stream)
            for i in range(args.mfma_probe_launches):
                fa.flat_attn_mfma_probe(sink, iters, rnd, stream)
                evs[i + 1].record(stream)
            torch.cuda.synchronize()
            tail = max(1, args.mfma_probe_launches // 4)  # the last quarter: clocks have settled
            ms = evs[-tail - 1].elapsed_time(evs[-1]) / tail
            probe[name] = round(fa.flat_attn_mfma_probe_flops(iters) / (ms * 1e-3) / 1e12, 1)
        probe["fused_vs_random_operand_mfma"] = round(kernel_tflops / probe["random_operands_tflops"], 4)

    cpu = None
    if args.cpu_rows_per_head > 0:
        import oracle
        nrows = min(args.cpu_rows_per_head, w.N)
        rows = np.arange(0, w.N, w.N // nrows, dtype=np.int64)[:nrows]
        q64, k64, v64 = (x.astype(np.float64) for x in (q, k, v))
        t3 = time.perf_counter()
        ref = oracle.attention(q64, k64, v64, w.scale, w.mask, rows=rows)
        cpu_s = time.perf_counter() - t3
        if w.mask == 1:
            cpu_flops = 4.0 * w.B * w.H * w.d * float(np.sum(rows + 1))
        else:
            cpu_flops = 4.0 * w.B * w.H * rows.size * w.N * w.d
        got = out[:, :, torch.from_numpy(rows).cuda(), :].float().cpu().numpy().astype(np.float64)
        diff = np.abs(got - ref)
        cpu = {"value": round(cpu_flops / cpu_s / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.hw_threads(), "kind": "oracle",
               "sample": f"{rows.size} evenly spaced query rows of each of the {w.B * w.H} heads ({cpu_s:.2f} s, fp64)",
               "seconds": round(cpu_s, 3),
               "seconds_all_rows_extrapolated": round(cpu_s * (w.flops_useful / cpu_flops), 1),
               "gpu_vs_oracle_max_abs": float(diff.max()), "gpu_vs_oracle_mean_rel": float(diff.sum() / np.abs(ref).sum())}

    peak = PEAK_BF16_TFLOPS if is_bf16 else PEAK_F32_TFLOPS
    rec = {
        "metric": METRIC,
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if is_bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "mask": "causal" if w.mask else "none",
                   "scale": w.scale, "flops_per_step": flops, "flops_nominal": w.flops_nominal},
        "pct_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2) if is_bf16 else None,
        "roofline": {"bound": "mfma", "achieved": round(kernel_tflops, 2), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(kernel_tflops / peak, 4), "kernel_ms": round(kernel_ms, 5),
                     "kernel_ms_median": round(per_launch[len(per_launch) // 2], 5), "kernel_ms_min": round(per_launch[0], 5),
                     "traffic": None if traffic is None else traffic.get("fused_bytes_per_launch")},
        "hbm_bytes": {"fused_algorithmic": fused_alg_bytes, "unfused_algorithmic": unfused_alg_bytes,
                      "fused_measured": None if traffic is None else traffic.get("fused_bytes_per_launch"),
                      "unfused_measured": None if traffic is None else traffic.get("unfused_bytes_per_launch")},
        "unfused": unfused,
        "mfma_probe": probe,
        "cpu_baseline": cpu,
    }
    print(json.dumps(rec))
    return 0


if __name__ == "__main__":
    sys.exit(main())
