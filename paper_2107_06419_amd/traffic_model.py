"""Closed-form traffic and buffer model of the attention block: what the paper's analysis predicts, what this
library's kernels should move, and how both compare with measured rocprofv3 byte counters.

Pure host arithmetic (no GPU, no kernels):  python -m paper_2107_06419_amd.traffic_model  prints the
prediction-versus-measurement table for the rocprofv3 traffic summaries under profiles/.

Paper side
  * on-chip buffer needed by the fused Logit-softmax-Attend tile at each execution granularity
    (section 5.3, "On-chip buffer requirement", and the table of buffer requirements per granularity);
  * operational intensity of the single Logit / Attend operators and of the fused pair (section 3.1,
    "Challenge 1", and section 4.1).
Kernel side
  * on-chip bytes of one workgroup of the fused kernel (K/V ring in LDS plus register state), which unlike the
    paper's row-granularity tile does not grow with N because the row maximum and sum are running values;
  * off-chip bytes of the fused kernel: the algorithmic minimum (every tensor once), the no-reuse upper bound
    (every workgroup streams its K/V range from memory), and in between an L2 model (workgroups resident on
    one XCD at the same time share one pass over K/V);
  * off-chip bytes of the unfused baseline: the fp32 N x N intermediate crosses memory four times.
"""
from __future__ import annotations

import json
import os
from dataclasses import dataclass

# ----------------------------------------------------------------------------------------------------------
# Paper: buffer requirement per granularity, in tensor ELEMENTS (table of buffer requirements, section 5.3).
# Derivation stated there for the row granularity: the Logit operator holds its two operand tiles, R x d of Q
# and N x d of K, double-buffered; the Attend operator holds N x d of V and its R x d output, double-buffered;
# the R x N intermediate is held once (it never talks to off-chip memory).  The coarser granularities follow
# by taking all N rows (head), all H heads (batch) and all B batch entries (batched multi-head).


def buffer_elements_row(R: int, N: int, d: int) -> int:
    logit_operands = 2 * (R * d + N * d)
    attend_operands = 2 * (N * d + R * d)
    intermediate = R * N
    return logit_operands + attend_operands + intermediate


def buffer_elements_head(N: int, d: int) -> int:
    return buffer_elements_row(N, N, d)


def buffer_elements_batch(H: int, N: int, d: int) -> int:
    return H * buffer_elements_head(N, d)


def buffer_elements_multihead(B: int, H: int, N: int, d: int) -> int:
    return B * buffer_elements_batch(H, N, d)


def largest_row_granularity(buffer_elements: int, N: int, d: int) -> int:
    """Largest R whose row-granularity tile fits a buffer of that many elements (0 if even R = 1 does not):
    the knob the paper turns when the sequence grows against a fixed on-chip memory."""
    spare = buffer_elements - 4 * N * d
    return max(0, min(N, spare // (4 * d + N)))


# ----------------------------------------------------------------------------------------------------------
# Paper: operational intensity = operations / memory accesses (section 2.1), in MACs per element as the paper
# counts them.  Single Logit or Attend over B batches and H heads of size d (D = H d): B N^2 D operations
# against two B N D activations and one B H N^2 activation (section 3.1).  Fused pair: twice the operations,
# and only Q, K, V, O cross the boundary (section 4.1).


def intensity_single(B: int, H: int, N: int, d: int) -> float:
    D = H * d
    return (B * N * N * D) / (2 * B * N * D + B * H * N * N)


def intensity_fused(B: int, H: int, N: int, d: int) -> float:
    D = H * d
    return (2 * B * N * N * D) / (4 * B * N * D)


def logit_attend_share(N: int, D: int, ffn_multiple: int = 4) -> float:
    """Share of one attention block's multiply-accumulates that sits in the Logit and Attend operators: N^2 D each,
    against 4 N D^2 for the Q/K/V/O projections and 2 * ffn_multiple N D^2 for the two feed-forward layers
    (operator list of section 2).  The paper reports the measured runtime share of the two operators growing
    with the sequence length (section 7, block- and model-level discussion); the operation count reproduces it."""
    la = 2 * N * N * D
    rest = 4 * N * D * D + 2 * ffn_multiple * N * D * D
    return la / (la + rest)


# ----------------------------------------------------------------------------------------------------------
# This library's fused kernel.


@dataclass(frozen=True)
class TileShape:
    d: int
    rows_per_workgroup: int
    keys_per_tile: int
    wavefronts: int
    lds_stages: int
    workgroups_per_cu: int


DEFAULT_SHAPES = {64: TileShape(64, 256, 64, 4, 4, 2), 128: TileShape(128, 256, 64, 8, 3, 1)}
XCDS = 8
CUS_PER_XCD = 32


def kernel_lds_bytes(t: TileShape, elem: int = 2) -> int:
    """K tile and V tile per ring stage."""
    return t.lds_stages * 2 * t.keys_per_tile * t.d * elem


def kernel_register_state_bytes(t: TileShape) -> int:
    """Per workgroup, the state that the paper's tile would keep in its buffer: the Q rows (bf16) and the fp32
    output accumulator of every row, plus one 32-key block of logits / probabilities in flight per wavefront
    (fp32 logits of the current and next block, bf16 probabilities of the current and previous block)."""
    q = t.rows_per_workgroup * t.d * 2
    o = t.rows_per_workgroup * t.d * 4
    block = t.rows_per_workgroup * 32 * (4 + 4 + 2 + 2)
    return q + o + block


def fused_min_bytes(B: int, H: int, N: int, d: int, elem: int = 2) -> dict:
    t = B * H * N * d * elem
    return {"fetch": 3 * t, "write": t}


def _kv_rows_streamed(N: int, Br: int, Bc: int, causal: bool) -> int:
    """Key rows streamed by all row blocks of one head (tiles of Bc keys; causal blocks stop at their diagonal)."""
    total = 0
    for qt in range((N + Br - 1) // Br):
        kv_len = min(N, (qt + 1) * Br) if causal else N
        total += ((kv_len + Bc - 1) // Bc) * Bc
    return total


def fused_no_reuse_bytes(B: int, H: int, N: int, d: int, causal: bool, t: TileShape, elem: int = 2) -> dict:
    """Every workgroup fetches its whole K/V range from memory (no cache helps)."""
    kv = 2 * _kv_rows_streamed(N, t.rows_per_workgroup, t.keys_per_tile, causal) * d * elem
    q = N * d * elem
    return {"fetch": B * H * (q + kv), "write": B * H * N * d * elem}


def fused_l2_model_bytes(B: int, H: int, N: int, d: int, causal: bool, t: TileShape, elem: int = 2) -> dict:
    """Workgroups resident on one XCD at the same time and working on the same head walk K/V together, so one
    pass over that head's K/V fills the L2 for all of them.  The model replays the kernel's block order: each
    XCD executes its blocks in rounds of as many workgroups as it has slots, and every distinct head in a round
    costs one pass, as long as the round's longest row block needs (all N keys without a mask)."""
    slots = CUS_PER_XCD * t.workgroups_per_cu
    Br = t.rows_per_workgroup
    n_qtiles = (N + Br - 1) // Br
    heads = B * H
    n_blocks = heads * n_qtiles
    per_xcd = (n_blocks + XCDS - 1) // XCDS
    kv_rows = 0
    for x in range(XCDS):
        for start in range(0, per_xcd, slots):
            longest = {}  # head -> longest key range among its blocks of this round
            for r in range(start, min(start + slots, per_xcd)):
                if causal:
                    g = XCDS * r + x            # ranks dealt to the XCDs like cards, heaviest first
                    if g >= n_blocks:
                        continue
                    head, qt = g % heads, n_qtiles - 1 - g // heads
                    kv_len = min(N, (qt + 1) * Br)
                else:
                    logical = x * per_xcd + r   # contiguous range per XCD, head after head
                    if logical >= n_blocks:
                        continue
                    head, kv_len = logical // n_qtiles, N
                longest[head] = max(longest.get(head, 0), kv_len)
            kv_rows += sum(longest.values())
    q = heads * N * d * elem
    return {"fetch": q + 2 * kv_rows * d * elem, "write": heads * N * d * elem, "kv_passes_per_head": kv_rows / (heads * N)}


def unfused_bytes(B: int, H: int, N: int, d: int, causal: bool, elem: int = 2, single_read_softmax: bool = True) -> dict:
    """GEMM writes fp32 L; the row softmax reads it (twice if the row does not stay on chip) and writes it;
    the second GEMM reads it.  With the causal mask the first GEMM skips the 128 x 128 tiles above the diagonal
    and the softmax reads only the visible part of a row but writes all of it (the zeros)."""
    heads = B * H
    sq = N * N * 4
    t = N * d * elem
    if causal:
        nt = (N + 127) // 128
        visible_tiles = nt * (nt + 1) // 2
        gemm1_write = min(sq, visible_tiles * 128 * 128 * 4)
        softmax_read = (N * (N + 1) // 2) * 4
        nb = (N + 127) // 128
        gemm2_read = sum(min(N, ((i + 1) * 128 + 63) // 64 * 64) * min(128, N - i * 128) * 4 for i in range(nb))
    else:
        gemm1_write = sq
        softmax_read = sq
        gemm2_read = sq
    softmax_read *= 1 if single_read_softmax else 2
    fetch = heads * (2 * t + softmax_read + gemm2_read + t)
    write = heads * (gemm1_write + sq + t)
    return {"fetch": fetch, "write": write}


# ----------------------------------------------------------------------------------------------------------
# Comparison with measured counters (profiles/hbm_traffic_<workload>.json, written by rocprof_summary --traffic).


def measured(path: str) -> dict:
    with open(path) as f:
        j = json.load(f)
    fused = {k: v for k, v in j["kernels"].items() if "fwd_bf16_kernel" in k}
    unf = {k: v for k, v in j["kernels"].items() if "fwd_bf16_kernel" not in k}
    out = {"fused_fetch": sum(v["fetch_bytes"] for v in fused.values()), "fused_write": sum(v["write_bytes"] for v in fused.values())}
    if unf:
        out["unfused_fetch"] = sum(v["fetch_bytes"] for v in unf.values())
        out["unfused_write"] = sum(v["write_bytes"] for v in unf.values())
    return out


def comparison_rows(profile_dir: str):
    from . import synth
    rows = []
    for name, w in synth.WORKLOADS.items():
        path = os.path.join(profile_dir, f"hbm_traffic_{name}.json")
        if w.dtype != "bf16" or not os.path.exists(path):
            continue
        m = measured(path)
        t = DEFAULT_SHAPES[w.d]
        lo = fused_min_bytes(w.B, w.H, w.N, w.d)
        mid = fused_l2_model_bytes(w.B, w.H, w.N, w.d, bool(w.mask), t)
        hi = fused_no_reuse_bytes(w.B, w.H, w.N, w.d, bool(w.mask), t)
        u = unfused_bytes(w.B, w.H, w.N, w.d, bool(w.mask))
        rows.append({"workload": name, "measured": m, "fused_min": lo, "fused_l2_model": mid, "fused_no_reuse": hi, "unfused_model": u})
    return rows


def main() -> int:
    here = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    rows = comparison_rows(os.path.join(here, "profiles"))
    mb = lambda x: f"{x / 1e6:.1f}"
    print("| workload | fused FETCH measured | minimum | L2 model | no-reuse bound | fused WRITE measured | predicted | "
          "unfused FETCH+WRITE measured | predicted |")
    print("|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        m = r["measured"]
        unf_m = mb(m["unfused_fetch"] + m["unfused_write"]) if "unfused_fetch" in m else "-"
        print(f"| {r['workload']} | {mb(m['fused_fetch'])} | {mb(r['fused_min']['fetch'])} | {mb(r['fused_l2_model']['fetch'])} | "
              f"{mb(r['fused_no_reuse']['fetch'])} | {mb(m['fused_write'])} | {mb(r['fused_min']['write'])} | {unf_m} | "
              f"{mb(r['unfused_model']['fetch'] + r['unfused_model']['write'])} |")
    print("\n(all figures in MB = 1e6 bytes)")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
