#!/usr/bin/env python3
"""Benchmark of the fused attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one call of flat_attn_fwd (the whole fused Logit-softmax-Attend path) on one synthetic
batch of the named workload, inputs resident in HBM.  Prints ONE JSON line: whole-job throughput
in TFLOP/s (4*B*H*N^2*d flops per step; for a causal workload the useful 2*B*H*N*(N+1)*d), the
MFMA roofline of the fused kernel measured with HIP events inside the timed region, the unfused
baseline's time and HBM bytes for comparison, the instruction-mix ceiling probes, the other four
workloads in compact form, and the CPU oracle timed on a bounded sample.

Exit status: 0 = measured and within tolerance; 2 = more than one GPU asked for; 3 = no GPU;
4 = some output compared with the oracle broke the stated tolerance (the JSON line is still printed).
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
PEAK_HBM_GBPS = 8000.0     # published HBM3E bandwidth
METRIC = "fused attention TFLOP/s and % bf16 MFMA peak at N=16K,d=64; HBM bytes vs unfused"
# tolerances of the build: (max |dO|, sum|dO| / sum|O_ref|) over all compared elements, plus a bound on
# sum|dO| / sum|O_ref| taken row by row, so that one wrong row or tile cannot hide in the aggregate
TOL = {"bf16": (2e-2, 5e-3, 3e-2), "f32": (1e-4, 1e-4, 1e-3)}
ROW_FLOOR = {"bf16": 1e-4, "f32": 1e-6}  # absolute slack per element of a row, for rows whose reference is all but zero
PREWARM_MS = 50.0          # GPU time spent on the fused kernel before anything is timed: clocks settle in about 25 ms


def compare(got, ref, dtype):
    """Errors of `got` [..., rows, d] against the oracle's `ref`, and whether they are within tolerance."""
    import numpy as np
    diff = np.abs(got - ref)
    max_abs = float(diff.max())
    mean_rel = float(diff.sum() / max(np.abs(ref).sum(), 1e-300))
    row_rel = float((np.maximum(diff.sum(axis=-1) - got.shape[-1] * ROW_FLOOR[dtype], 0.0) / np.maximum(np.abs(ref).sum(axis=-1), 1e-300)).max())
    t = TOL[dtype]
    ok = bool(np.isfinite(got).all() and max_abs <= t[0] and mean_rel <= t[1] and row_rel <= t[2])
    return {"max_abs": max_abs, "mean_rel": mean_rel, "worst_row_rel": row_rel, "ok": ok}


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
    ap.add_argument("--mix-probe-launches", type=int, default=12, help="launches of each instruction-mix probe level (0 = skip)")
    ap.add_argument("--others", type=int, default=1, help="1 = also time and check the other four workloads, compactly (0 = skip)")
    ap.add_argument("--other-rows-per-head", type=int, default=256, help="oracle sample per head for the other workloads")
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

    def prewarm(fn, ms=PREWARM_MS):
        """Launch fn until `ms` of GPU time have passed (HIP events); returns the GPU milliseconds spent."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        spent = 0.0
        while spent < ms:
            e0.record(stream)
            for _ in range(8):
                fn()
            e1.record(stream)
            e1.synchronize()
            spent += e0.elapsed_time(e1)
        return spent

    clock_prewarm_ms = prewarm(step)
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

    # the fused step's instruction mix on synthetic data: registers only, then with the kernel's data movement
    # added rung by rung (level 3 has the structure of the fused kernel's main loop)
    mix = None
    if args.mix_probe_launches > 0 and is_bf16:
        sink = torch.empty(fa.flat_attn_mix_probe_sink_bytes() // 4, dtype=torch.float32, device="cuda")
        src = torch.randn(fa.flat_attn_mix_probe_src_bytes() // 2, device="cuda").to(torch.bfloat16)
        iters = 500
        mix = {}
        names = ("registers_only_tflops", "plus_lds_operand_reads_tflops", "plus_tile_barrier_tflops", "plus_global_to_lds_streaming_tflops")
        for level, name in enumerate(names):
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.mix_probe_launches + 1)]
            evs[0].record(stream)
            for i in range(args.mix_probe_launches):
                fa.flat_attn_mix_probe(sink, src, level, iters, stream)
                evs[i + 1].record(stream)
            torch.cuda.synchronize()
            tail = max(1, args.mix_probe_launches // 2)
            ms = evs[-tail - 1].elapsed_time(evs[-1]) / tail
            mix[name] = round(fa.flat_attn_mix_probe_flops(iters) / (ms * 1e-3) / 1e12, 1)
        prewarm(step, 10.0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(20):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        again = flops / (e0.elapsed_time(e1) / 20 * 1e-3) / 1e12  # the fused kernel right after the probes: same clocks
        mix["fused_kernel_tflops_same_minute"] = round(again, 1)
        mix["fused_vs_registers_only"] = round(again / mix[names[0]], 4)
        mix["fused_vs_full_structure"] = round(again / mix[names[3]], 4)
        mix["registers_only_frac_of_peak"] = round(mix[names[0]] / PEAK_BF16_TFLOPS, 4)
        del sink, src

    parity_ok = True
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
        step()
        torch.cuda.synchronize()
        got = out[:, :, torch.from_numpy(rows).cuda(), :].float().cpu().numpy().astype(np.float64)
        cmp_ = compare(got, ref, w.dtype)
        parity_ok = parity_ok and cmp_["ok"]
        cpu = {"value": round(cpu_flops / cpu_s / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.hw_threads(), "kind": "oracle",
               "sample": f"{rows.size} evenly spaced query rows of each of the {w.B * w.H} heads ({cpu_s:.2f} s, fp64)",
               "seconds": round(cpu_s, 3),
               "seconds_all_rows_extrapolated": round(cpu_s * (w.flops_useful / cpu_flops), 1),
               "gpu_vs_oracle_max_abs": cmp_["max_abs"], "gpu_vs_oracle_mean_rel": cmp_["mean_rel"],
               "gpu_vs_oracle_worst_row_rel": cmp_["worst_row_rel"], "within_tolerance": cmp_["ok"],
               "tolerance": {"max_abs": TOL[w.dtype][0], "mean_rel": TOL[w.dtype][1], "worst_row_rel": TOL[w.dtype][2]}}

    # the other workloads of the benchmark set, compactly: time of the fused kernel and a sampled oracle check
    others = None
    if args.others:
        import oracle
        others = []
        del dq, dk, dv, out
        for name, ow in synth.WORKLOADS.items():
            if name == w.name:
                continue
            obf = ow.dtype == "bf16"
            oq, ok_, ov = synth.make_qkv(ow)

            def odev(x):
                if not obf:
                    return torch.from_numpy(np.ascontiguousarray(x)).cuda()
                return torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda().view(torch.bfloat16)

            tq, tk, tv = odev(oq), odev(ok_), odev(ov)
            to = torch.empty_like(tq)
            ofwd = fa.flat_attn_fwd if obf else fa.flat_attn_fwd_f32

            def ostep():
                ofwd(tq, tk, tv, to, ow.scale, ow.mask, stream)

            prewarm(ostep, 30.0)
            n = 30
            es = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for a, b in es:
                a.record(stream)
                ostep()
                b.record(stream)
            torch.cuda.synchronize()
            ts = sorted(a.elapsed_time(b) for a, b in es)
            med = ts[n // 2]
            nrows = min(args.other_rows_per_head, ow.N)
            rows = np.unique(np.concatenate([np.arange(0, ow.N, max(1, ow.N // nrows), dtype=np.int64)[:nrows],
                                             np.array([0, ow.N - 1], dtype=np.int64)]))
            ref = oracle.attention(oq.astype(np.float64), ok_.astype(np.float64), ov.astype(np.float64), ow.scale, ow.mask, rows=rows)
            got = to[:, :, torch.from_numpy(rows).cuda(), :].float().cpu().numpy().astype(np.float64)
            c_ = compare(got, ref, ow.dtype)
            parity_ok = parity_ok and c_["ok"]
            opeak = PEAK_BF16_TFLOPS if obf else PEAK_F32_TFLOPS
            otf = ow.flops_useful / (med * 1e-3) / 1e12
            others.append({"workload": name, "dtype": ow.dtype, "mask": "causal" if ow.mask else "none",
                           "ms_median": round(med, 5), "ms_min": round(ts[0], 5), "tflops_useful": round(otf, 2),
                           "frac_of_peak": round(otf / opeak, 4), "rows_checked_per_head": int(rows.size),
                           "max_abs": c_["max_abs"], "mean_rel": c_["mean_rel"], "worst_row_rel": c_["worst_row_rel"],
                           "within_tolerance": c_["ok"]})
            del tq, tk, tv, to, oq, ok_, ov

    # few query rows over a long cache (B=1, H=16, Nq new positions over 65536 keys, causal): bound by reading K and V
    # once from HBM, not by the matrix units; one workgroup per row block against the split-keys form
    short = None
    if args.others:
        import oracle
        short = []
        sB, sH, sNk, sd = 1, 16, 65536, 64

        def rounded(shape, seed, tid):
            x = synth.tensor_f32(shape, seed, tid, "normal", 1.0)
            return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x)).reshape(shape)

        def dev16(x):
            return torch.from_numpy(synth.f32_to_bf16_bits(x).reshape(x.shape).view(np.int16)).cuda().view(torch.bfloat16)

        hk, hv = rounded((sB, sH, sNk, sd), 4242, 1), rounded((sB, sH, sNk, sd), 4242, 2)
        tk, tv = dev16(hk), dev16(hv)
        for sNq in (1, 64, 256):
            hq = rounded((sB, sH, sNq, sd), 4242 + sNq, 0)
            tq = dev16(hq)
            to = torch.empty_like(tq)
            ws = torch.empty(fa.flat_attn_fwd_splitkv_workspace_bytes(sB, sH, sNq, sNk, sd, 0) // 4, dtype=torch.float32, device="cuda")
            ref = oracle.attention_cross(hq.astype(np.float64), hk.astype(np.float64), hv.astype(np.float64), 0.125, 1)
            alg_bytes = 2 * sB * sH * sNk * sd * 2 + 2 * sB * sH * sNq * sd * 2  # K, V once; Q, O
            entry = {"Nq": sNq, "Nk": sNk, "H": sH, "d": sd, "mask": "causal", "algorithmic_hbm_bytes": alg_bytes,
                     "n_splits": fa.flat_attn_fwd_splitkv_splits(sB, sH, sNq, sNk, sd, 0)}
            for label, fn in (("one_workgroup_per_row_block", lambda: fa.flat_attn_fwd_cross(tq, tk, tv, to, 0.125, 1, None, stream)),
                              ("split_keys", lambda: fa.flat_attn_fwd_splitkv(tq, tk, tv, to, 0.125, 1, None, 0, ws, stream))):
                prewarm(fn, 20.0)
                n = 20
                es = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
                for a, b in es:
                    a.record(stream)
                    fn()
                    b.record(stream)
                torch.cuda.synchronize()
                ts = sorted(a.elapsed_time(b) for a, b in es)
                c_ = compare(to.float().cpu().numpy().astype(np.float64), ref, "bf16")
                parity_ok = parity_ok and c_["ok"]
                gbps = alg_bytes / (ts[n // 2] * 1e-3) / 1e9
                entry[label] = {"ms_median": round(ts[n // 2], 5), "ms_min": round(ts[0], 5), "hbm_gbps": round(gbps, 1),
                                "frac_of_hbm_peak": round(gbps / PEAK_HBM_GBPS, 4), "mean_rel": c_["mean_rel"],
                                "worst_row_rel": c_["worst_row_rel"], "within_tolerance": c_["ok"]}
            short.append(entry)
        del tk, tv

    peak = PEAK_BF16_TFLOPS if is_bf16 else PEAK_F32_TFLOPS
    rec = {
        "metric": METRIC,
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "clock_prewarm_ms": round(clock_prewarm_ms, 1),
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
        "mix_ceiling": mix,
        "cpu_baseline": cpu,
        "other_workloads": others,
        "short_query_over_long_cache": short,
        "parity_ok": parity_ok,
    }
    print(json.dumps(rec))
    if not parity_ok:
        print("bench.py: an output compared with the oracle is outside the stated tolerance", file=sys.stderr)
        return 4
    return 0


if __name__ == "__main__":
    sys.exit(main())
