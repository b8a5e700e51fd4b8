"""Seeded synthetic Q/K/V tensors for the attention workloads.

This module only produces inputs.  It holds none of the attention arithmetic
and is the single piece of code shared by the GPU tests, the benchmark and the
CPU oracle's tests.  It depends on numpy alone.

Generator: a counter-based hash.  Element `i` of tensor `t` under seed `s` is a
pure function of (s, t, i), so any slice can be regenerated independently and
the result does not depend on chunking, thread count or library version:

    x  = splitmix64-style finaliser of (s, t, i)
    u1 = (high 32 bits of x + 1) / 2^32      in (0, 1]
    u2 = (low  32 bits of x)     / 2^32      in [0, 1)
    normal  = sqrt(-2 ln u1) * cos(2 pi u2)  (Box-Muller, computed in float64)
    uniform = 2 * ((x >> 11) / 2^53) - 1     in [-1, 1)

Values are rounded once to float32 and, for bf16 workloads, once more to
bfloat16 with round-to-nearest-even; the bf16 bit patterns are returned as
uint16 so no tensor library is needed here.

The five workloads mirror the shapes the paper sweeps (BERT-base-like heads,
sequence lengths 512 ... 64K, Section 6 "Workloads"); the paper evaluates on
shapes only, so random tensors of those shapes stand in for its models.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

TENSOR_Q, TENSOR_K, TENSOR_V = 0, 1, 2

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _hash64(seed: int, tensor_id: int, idx: np.ndarray) -> np.ndarray:
    """64-bit mix of (seed, tensor_id, idx); idx is a uint64 array."""
    with np.errstate(over="ignore"):
        base = np.uint64((seed * 0xD6E8FEB86659FD93 + (tensor_id + 1) * 0xA0761D6478BD642F) & 0xFFFFFFFFFFFFFFFF)
        x = idx * _GOLDEN + base
        x ^= x >> np.uint64(30)
        x *= _M1
        x ^= x >> np.uint64(27)
        x *= _M2
        x ^= x >> np.uint64(31)
    return x


def _fill(out: np.ndarray, seed: int, tensor_id: int, dist: str, mult: float, start: int = 0) -> None:
    n = out.size
    flat = out.reshape(-1)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        idx = np.arange(start + lo, start + hi, dtype=np.uint64)
        x = _hash64(seed, tensor_id, idx)
        if dist == "normal":
            u1 = ((x >> np.uint64(32)).astype(np.float64) + 1.0) * (1.0 / 4294967296.0)
            u2 = (x & np.uint64(0xFFFFFFFF)).astype(np.float64) * (1.0 / 4294967296.0)
            v = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        elif dist == "uniform":
            v = 2.0 * ((x >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)) - 1.0
        else:
            raise ValueError(f"unknown distribution {dist!r}")
        flat[lo:hi] = (v * mult).astype(np.float32)


def tensor_f32(shape, seed: int, tensor_id: int, dist: str = "normal", mult: float = 1.0) -> np.ndarray:
    """float32 tensor of `shape`, element i (row-major) = f(seed, tensor_id, i)."""
    out = np.empty(shape, dtype=np.float32)
    _fill(out, seed, tensor_id, dist, mult)
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    if np.any((u & np.uint32(0x7F800000)) == np.uint32(0x7F800000)):
        raise ValueError("non-finite value in synthetic input")
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32, exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: str          # "bf16" or "f32": storage type of Q, K, V, O
    mask: int           # 0 = none, 1 = causal (key j visible to query i iff j <= i)
    scale: float        # float32 value handed across the C ABI
    qk_mult: float      # Q, K ~ qk_mult * N(0, 1)
    v_dist: str         # "normal" or "uniform" (U[-1, 1))
    seed: int

    @property
    def shape(self):
        return (self.B, self.H, self.N, self.d)

    @property
    def flops_nominal(self) -> float:
        return 4.0 * self.B * self.H * float(self.N) ** 2 * self.d

    @property
    def flops_useful(self) -> float:
        if self.mask == 1:
            return 2.0 * self.B * self.H * float(self.N) * (self.N + 1) * self.d
        return self.flops_nominal


_SEED0 = 20210706


def _f32(x: float) -> float:
    return float(np.float32(x))


WORKLOADS = {
    # BERT-base-shaped heads, fp32, finishes in seconds on the CPU oracle
    "cfg0_bert_base_f32": Workload("cfg0_bert_base_f32", 1, 12, 512, 64, "f32", 0, _f32(1.0 / 8.0), 1.0, "normal", _SEED0 + 0),
    # encoder batch
    "cfg1_encoder_4k": Workload("cfg1_encoder_4k", 8, 16, 4096, 64, "bf16", 0, _f32(1.0 / 8.0), 1.0, "normal", _SEED0 + 1),
    # headline: long sequence
    "cfg2_long_16k": Workload("cfg2_long_16k", 1, 16, 16384, 64, "bf16", 0, _f32(1.0 / 8.0), 1.0, "normal", _SEED0 + 2),
    # wide heads, peaky softmax, causal
    "cfg3_wide_causal_8k": Workload("cfg3_wide_causal_8k", 2, 8, 8192, 128, "bf16", 1, _f32(1.0 / np.sqrt(128.0)), 2.0, "uniform", _SEED0 + 3),
    # extreme length
    "cfg4_extreme_64k": Workload("cfg4_extreme_64k", 1, 8, 65536, 64, "bf16", 0, _f32(1.0 / 8.0), 1.0, "normal", _SEED0 + 4),
}


def make_qkv(w: Workload):
    """Q, K, V for a workload as float32 arrays holding the exact stored values.

    For a bf16 workload the float32 values are exactly representable in bf16
    (already rounded), so `f32_to_bf16_bits` on them is lossless and widening
    to float64 for the oracle is exact.
    """
    vm = 1.0
    q = tensor_f32(w.shape, w.seed, TENSOR_Q, "normal", w.qk_mult)
    k = tensor_f32(w.shape, w.seed, TENSOR_K, "normal", w.qk_mult)
    v = tensor_f32(w.shape, w.seed, TENSOR_V, w.v_dist, vm)
    if w.dtype == "bf16":
        q = bf16_bits_to_f32(f32_to_bf16_bits(q)).reshape(w.shape)
        k = bf16_bits_to_f32(f32_to_bf16_bits(k)).reshape(w.shape)
        v = bf16_bits_to_f32(f32_to_bf16_bits(v)).reshape(w.shape)
    return q, k, v


def custom(name: str, B: int, H: int, N: int, d: int, dtype: str = "bf16", mask: int = 0,
           scale: float | None = None, qk_mult: float = 1.0, v_dist: str = "normal", seed: int = 1) -> Workload:
    """A workload of arbitrary shape with the same recipe (for tests)."""
    if scale is None:
        scale = 1.0 / float(np.sqrt(float(d)))
    return Workload(name, B, H, N, d, dtype, mask, _f32(scale), qk_mult, v_dist, seed)


def random_block_pattern(n_lists: int, n_key_tiles: int, keep: float, seed: int, at_least_one: bool = True):
    """Seeded random block pattern in CSR form: for each of `n_lists` row blocks, every key tile is kept with
    probability `keep` (counter-based: tile t of list r depends on (seed, r, t) only).  Returns (offsets int64
    [n_lists + 1], ids int64, ascending within a list).  With `at_least_one`, an otherwise empty list keeps tile
    (r mod n_key_tiles)."""
    u = tensor_f32((n_lists, n_key_tiles), seed, 7, "uniform", 1.0)  # uniform in [-1, 1)
    kept = (u.astype(np.float64) + 1.0) * 0.5 < keep
    if at_least_one:
        for r in np.flatnonzero(~kept.any(axis=1)):
            kept[r, r % n_key_tiles] = True
    counts = kept.sum(axis=1)
    offsets = np.zeros(n_lists + 1, dtype=np.int64)
    np.cumsum(counts, out=offsets[1:])
    ids = np.nonzero(kept)[1].astype(np.int64)
    return offsets, ids
