"""Shared helpers of the GPU parity tests: move seeded inputs to the device, run an entry point
through the C ABI binding, evaluate the CPU oracle on the same values, and measure the error."""
import numpy as np

import oracle
from paper_2107_06419_amd import synth

# Tolerances (the build's stated target): bf16 path max|dO| <= 2e-2 and sum|dO|/sum|O_ref| <= 5e-3;
# fp32 path <= 1e-4 on both.
TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-4, 1e-4)}
# Row by row (the last axis is the head dimension): sum_c|dO| <= rel * sum_c|O_ref| + d * floor.  The aggregate
# above does not move when a single row or tile is wrong; this bound does.  A correct bf16 row sits near 3e-3
# (rounding of O and of the probabilities), the worst of millions of rows below 1.5e-2.
ROW_TOL = {"bf16": (3e-2, 1e-4), "f32": (1e-3, 1e-6)}


def to_device(x_f32: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        bits = synth.f32_to_bf16_bits(x_f32).reshape(x_f32.shape)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x_f32)).cuda()


def to_host_f64(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def errors(got: np.ndarray, ref: np.ndarray):
    diff = np.abs(got - ref)
    return float(diff.max()), float(diff.sum() / max(np.abs(ref).sum(), 1e-300))


def check_close(got, ref, dtype, what=""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs, mean_rel = errors(got, ref)
    tol_abs, tol_rel = TOL[dtype]
    assert max_abs <= tol_abs and mean_rel <= tol_rel, f"{what}: max|dO|={max_abs:.3e} (<= {tol_abs}), mean rel={mean_rel:.3e} (<= {tol_rel})"
    row_rel, row_floor = ROW_TOL[dtype]
    excess = np.abs(got - ref).sum(axis=-1) - (row_rel * np.abs(ref).sum(axis=-1) + got.shape[-1] * row_floor)
    worst = np.unravel_index(int(np.argmax(excess)), excess.shape)
    assert excess[worst] <= 0.0, (f"{what}: row {worst} is off by sum|dO|={np.abs(got - ref)[worst].sum():.3e} against "
                                  f"sum|O_ref|={np.abs(ref)[worst].sum():.3e} (row bound {row_rel})")
    return max_abs, mean_rel


def sample_rows(N: int, n_random: int, seed: int, tiles=(32, 64, 128, 256)) -> np.ndarray:
    """Query rows for sampled comparison: first, last, both sides of tile boundaries, plus random ones."""
    rows = {0, N - 1}
    for t in tiles:
        for mult in (1, 2, 3, N // t // 2, N // t - 1):
            for delta in (-1, 0, 1):
                r = mult * t + delta
                if 0 <= r < N:
                    rows.add(r)
    rng = np.random.default_rng(seed)
    rows.update(int(r) for r in rng.integers(0, N, size=n_random))
    return np.array(sorted(rows), dtype=np.int64)


def oracle_rows(w: synth.Workload, q, k, v, rows=None):
    return oracle.attention(q, k, v, w.scale, w.mask, rows=rows)
