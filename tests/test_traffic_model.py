"""The traffic / buffer model against what the paper prints (tests/golden), against itself where the paper's
table rows must agree with each other, against the tile table compiled into the library, and against the
measured rocprofv3 byte counts committed under profiles/."""
import json
import os
import random

import pytest

import paper_2107_06419_amd as fa
from paper_2107_06419_amd import synth
from paper_2107_06419_amd import traffic_model as tm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")


def poly(monomials, env):
    total = 0
    for coeff, factors in monomials:
        term = coeff
        for f in factors:
            term *= env[f]
        total += term
    return total


def random_envs(n=25):
    rng = random.Random(7)
    for _ in range(n):
        B, H, N, d = rng.randint(1, 9), rng.randint(1, 17), rng.randint(1, 5000), rng.choice([16, 64, 80, 128])
        yield dict(B=B, H=H, N=N, d=d, D=H * d, R=rng.randint(1, N))


def test_buffer_requirements_match_the_papers_table():
    table = json.load(open(os.path.join(GOLDEN, "buffer_requirement_table.json")))
    for e in random_envs():
        assert tm.buffer_elements_row(e["R"], e["N"], e["d"]) == poly(table["R-Gran"], e)
        assert tm.buffer_elements_head(e["N"], e["d"]) == poly(table["H-Gran"], e)
        assert tm.buffer_elements_batch(e["H"], e["N"], e["d"]) == poly(table["B-Gran"], e)
        assert tm.buffer_elements_multihead(e["B"], e["H"], e["N"], e["d"]) == poly(table["M-Gran"], e)


def test_the_papers_table_rows_agree_with_each_other():
    """Independent of the model: a head tile is the row tile with R = N, a batch tile is H head tiles, and so on."""
    table = json.load(open(os.path.join(GOLDEN, "buffer_requirement_table.json")))
    for e in random_envs():
        assert poly(table["R-Gran"], dict(e, R=e["N"])) == poly(table["H-Gran"], e)
        assert e["H"] * poly(table["H-Gran"], e) == poly(table["B-Gran"], e)
        assert e["B"] * poly(table["B-Gran"], e) == poly(table["M-Gran"], e)


def test_largest_row_granularity_is_the_boundary():
    for e in random_envs():
        N, d = e["N"], e["d"]
        budget = tm.buffer_elements_row(e["R"], N, d)
        R = tm.largest_row_granularity(budget, N, d)
        assert R >= e["R"] and tm.buffer_elements_row(R, N, d) <= budget
        assert R == N or tm.buffer_elements_row(R + 1, N, d) > budget
    assert tm.largest_row_granularity(10, 4096, 64) == 0


def test_operational_intensity_matches_the_paper():
    g = json.load(open(os.path.join(GOLDEN, "operational_intensity.json")))
    for e in random_envs():
        want = poly(g["single_operations"], e) / poly(g["single_accesses"], e)
        assert tm.intensity_single(e["B"], e["H"], e["N"], e["d"]) == pytest.approx(want, rel=1e-12)
        # fused: both operators' work over Q, K, V, O only = N / 2, independent of d, B and H
        assert tm.intensity_fused(e["B"], e["H"], e["N"], e["d"]) == pytest.approx(e["N"] / 2, rel=1e-12)
    # long sequences: the single operator saturates at d (the N^2 term dominates), the fused pair keeps growing
    assert tm.intensity_single(1, 16, 1 << 20, 64) == pytest.approx(64, rel=1e-3)
    assert tm.intensity_fused(1, 16, 1 << 20, 64) / tm.intensity_single(1, 16, 1 << 20, 64) > 8000


def test_default_shapes_agree_with_the_library_table():
    for d, t in tm.DEFAULT_SHAPES.items():
        lib = fa.flat_attn_tile_shape_get(d, 0).as_dict()
        assert (lib["rows_per_workgroup"], lib["keys_per_tile"], lib["wavefronts"], lib["lds_stages"]) == \
               (t.rows_per_workgroup, t.keys_per_tile, t.wavefronts, t.lds_stages)
        assert lib["lds_bytes"] == tm.kernel_lds_bytes(t)
        assert t.workgroups_per_cu == min(160 * 1024 // lib["lds_bytes"], 8 // t.wavefronts)
        # on-chip state of a workgroup is independent of N, unlike the paper's R x N slab: at N = 64K the paper's
        # row tile of the same R needs two orders of magnitude more
        ours = tm.kernel_lds_bytes(t) + tm.kernel_register_state_bytes(t)
        assert tm.kernel_lds_bytes(t) <= 160 * 1024 and tm.kernel_register_state_bytes(t) <= 512 * 1024  # one CU's LDS / registers
        assert 2 * tm.buffer_elements_row(t.rows_per_workgroup, 65536, d) > 100 * ours


def test_fused_byte_models_are_ordered_and_scale_linearly():
    for w in synth.WORKLOADS.values():
        if w.dtype != "bf16":
            continue
        t = tm.DEFAULT_SHAPES[w.d]
        lo = tm.fused_min_bytes(w.B, w.H, w.N, w.d)
        mid = tm.fused_l2_model_bytes(w.B, w.H, w.N, w.d, bool(w.mask), t)
        hi = tm.fused_no_reuse_bytes(w.B, w.H, w.N, w.d, bool(w.mask), t)
        assert lo["fetch"] <= mid["fetch"] * (2.0 if w.mask else 1.0)  # a causal pass may stop short of N
        assert mid["fetch"] <= hi["fetch"]
        assert lo["write"] == mid["write"] == hi["write"] == w.B * w.H * w.N * w.d * 2
    # minimum traffic doubles with N; the unfused intermediate quadruples
    a, b = tm.fused_min_bytes(1, 16, 8192, 64), tm.fused_min_bytes(1, 16, 16384, 64)
    assert b["fetch"] == 2 * a["fetch"] and b["write"] == 2 * a["write"]
    ua, ub = tm.unfused_bytes(1, 16, 8192, 64, False), tm.unfused_bytes(1, 16, 16384, 64, False)
    assert (ub["write"] - b["write"]) == 4 * (ua["write"] - a["write"])
    # the 16 bytes per logit of the unfused path: write, read, write, read of an fp32 value
    n2 = 16 * 16384 * 16384
    assert ub["fetch"] + ub["write"] == 16 * n2 + 4 * 16 * 16384 * 64 * 2
    # brute-force count of the no-reuse bound on a tiny causal problem
    t = tm.TileShape(64, 256, 64, 4, 4, 2)
    rows = sum(-(-min(1000, (qt + 1) * 256) // 64) * 64 for qt in range(4))
    assert tm.fused_no_reuse_bytes(1, 1, 1000, 64, True, t)["fetch"] == 1000 * 128 + 2 * rows * 128


def test_measured_traffic_is_bracketed_by_the_model():
    rows = tm.comparison_rows(os.path.join(ROOT, "profiles"))
    assert {r["workload"] for r in rows} >= {"cfg1_encoder_4k", "cfg2_long_16k", "cfg3_wide_causal_8k", "cfg4_extreme_64k"}
    for r in rows:
        m = r["measured"]
        # the only off-chip write of the fused kernel is O
        assert m["fused_write"] == pytest.approx(r["fused_min"]["write"], rel=0.01)
        # reads: at least the L2 model's (up to counter noise), at most twice it, and nowhere near the no-reuse bound
        assert 0.95 * r["fused_l2_model"]["fetch"] <= m["fused_fetch"] <= 2.0 * r["fused_l2_model"]["fetch"]
        assert m["fused_fetch"] < 0.15 * r["fused_no_reuse"]["fetch"]
        if "unfused_fetch" in m:
            tot, model = m["unfused_fetch"] + m["unfused_write"], r["unfused_model"]["fetch"] + r["unfused_model"]["write"]
            assert model <= tot * 1.02 and tot <= 1.35 * model
            assert tot > 50 * (m["fused_fetch"] + m["fused_write"])


def test_logit_attend_share_follows_the_papers_runtime_shares():
    """The paper gives measured runtime shares; operation counts should land within a few points of them (the
    other operators run closer to peak than Logit/Attend do, so the measured share is the slightly larger one)."""
    g = json.load(open(os.path.join(GOLDEN, "logit_attend_runtime_share.json")))
    for N, pct in zip(g["sequence_lengths"], g["runtime_share_percent"]):
        share = 100.0 * tm.logit_attend_share(N, 768)
        assert pct - 3.0 <= share <= pct + 0.5, (N, share, pct)
    assert tm.logit_attend_share(1, 768) < 1e-3 and tm.logit_attend_share(1 << 24, 768) > 0.999
