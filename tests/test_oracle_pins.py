"""Pins for the CPU oracle: what the paper's definition and the mathematics fix.

The paper (section 2, steps 2-4) defines Logit / row-Softmax / Attend and states
that the fused dataflow leaves the function unchanged, but prints no numeric
example.  So the oracle is pinned by
  * a hand-worked example with rational probabilities (tests/golden/),
  * brute force on tiny shapes written without max-subtraction,
  * closed forms, and
  * invariants of softmax attention.
Every pin is a function of an `attn(Q, K, V, scale, mask)` callable, so the same
pins are also run against deliberately wrong implementations (mutants) to show
that each plausible mistake trips at least one of them.
"""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2107_06419_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def oracle_attn(Q, K, V, scale, mask):
    return oracle.attention(Q, K, V, scale, mask)


def rnd(shape, seed, tid=0, dist="normal", mult=1.0):
    return synth.tensor_f32(shape, seed, tid, dist, mult).astype(np.float64)


# ----------------------------------------------------------------------------- pins
def pin_hand_example(attn):
    g = json.load(open(os.path.join(GOLDEN, "hand_example_3x2.json")))
    sym = {"ln2": math.log(2.0), "ln3": math.log(3.0)}
    Q = np.array([[sym.get(x, x) for x in row] for row in g["Q_exact"]], dtype=np.float64)[None, None]
    K = np.array(g["K"], dtype=np.float64)[None, None]
    V = np.array(g["V"], dtype=np.float64)[None, None]
    for mask, key in ((0, "O_none_rational"), (1, "O_causal_rational")):
        want = np.array([[float(Fraction(*x)) for x in row] for row in g[key]])
        got = attn(Q, K, V, g["scale"], mask)[0, 0]
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)
    # same numbers through a non-unit scale: (2Q) * 0.5
    got = attn(2.0 * Q, K, V, 0.5, 0)[0, 0]
    want = np.array([[float(Fraction(*x)) for x in row] for row in g["O_none_rational"]])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


def _brute(Q, K, V, scale, mask):
    """Per output element, directly: sum_j exp(L_ij) V_jc / sum_j exp(L_ij); no max-subtraction, long double."""
    B, H, N, d = Q.shape
    ld = np.longdouble
    O = np.zeros((B, H, N, d))
    for b in range(B):
        for h in range(H):
            for i in range(N):
                for c in range(d):
                    num, den = ld(0), ld(0)
                    for j in range(N):
                        if mask == 1 and j > i:
                            continue
                        lij = ld(0)
                        for k in range(d):
                            lij += ld(Q[b, h, i, k]) * ld(K[b, h, j, k])
                        w = np.exp(lij * ld(scale))
                        num += w * ld(V[b, h, j, c])
                        den += w
                    O[b, h, i, c] = float(num / den)
    return O


def pin_brute_force(attn):
    for seed, (B, H, N, d) in enumerate([(1, 1, 1, 1), (1, 1, 2, 1), (2, 3, 5, 3), (1, 2, 8, 4), (2, 1, 7, 2), (1, 1, 3, 4)]):
        Q, K, V = (rnd((B, H, N, d), 100 + seed, t) for t in range(3))
        for mask in (0, 1):
            for scale in (1.0, 0.37):
                got = attn(Q, K, V, scale, mask)
                want = _brute(Q, K, V, scale, mask)
                np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def pin_uniform_logits(attn):
    B, H, N, d = 2, 2, 37, 5
    Q, K, V = (rnd((B, H, N, d), 7, t) for t in range(3))
    zero = np.zeros_like(K)
    for Qx, Kx in ((Q, zero), (zero, K)):
        got = attn(Qx, Kx, V, 0.3, 0)
        want = np.broadcast_to(V.mean(axis=2, keepdims=True), V.shape)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)
        got = attn(Qx, Kx, V, 0.3, 1)
        want = np.cumsum(V, axis=2) / np.arange(1, N + 1)[None, None, :, None]
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def pin_dominant_key(attn):
    B, H, N, d = 1, 2, 33, 4
    Q, K, V = (rnd((B, H, N, d), 11, t) for t in range(3))
    Q = np.abs(Q) + 0.5                      # every query has a positive first coordinate
    K = 0.01 * K
    jstar = 19
    K[:, :, jstar, :] = 0.0
    K[:, :, jstar, 0] = 200.0                # logit of key j* exceeds the others by >= 200*0.5 - small
    got = attn(Q, K, V, 1.0, 0)
    gap = 200.0 * 0.5 - 1.0
    bound = 2.0 * (N - 1) * math.exp(-gap) * np.abs(V).max()
    want = np.broadcast_to(V[:, :, jstar:jstar + 1, :], V.shape)
    assert np.abs(got - want).max() <= bound + 1e-15
    # two equal dominant keys with huge logits (stability): the mean of their value rows
    K[:, :, 3, :] = K[:, :, jstar, :]
    got = attn(Q, 10.0 * K, V, 1.0, 0)       # logits up to ~2000*|q| : exp() would overflow without max-subtraction
    want = 0.5 * (V[:, :, 3:4, :] + V[:, :, jstar:jstar + 1, :])
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, np.broadcast_to(want, V.shape), rtol=0, atol=1e-13)


def pin_constant_value_columns(attn):
    B, H, N, d = 1, 3, 29, 6
    Q, K = (rnd((B, H, N, d), 13, t) for t in range(2))
    col = np.arange(1, d + 1, dtype=np.float64) * 0.25
    V = np.broadcast_to(col, (B, H, N, d)).copy()
    for mask in (0, 1):
        np.testing.assert_allclose(attn(Q, K, V, 0.7, mask), V, rtol=0, atol=1e-14)


def pin_degenerate_rows(attn):
    Q, K, V = (rnd((2, 2, 9, 3), 17, t) for t in range(3))
    got = attn(Q, K, V, 0.5, 1)
    np.testing.assert_array_equal(got[:, :, 0, :], V[:, :, 0, :])           # causal row 0 sees key 0 only
    Q1, K1, V1 = (rnd((2, 2, 1, 3), 19, t) for t in range(3))
    for mask in (0, 1):
        np.testing.assert_array_equal(attn(Q1, K1, V1, 0.5, mask), V1)      # N = 1


def pin_permutation(attn):
    B, H, N, d = 2, 2, 31, 4
    Q, K, V = (rnd((B, H, N, d), 23, t) for t in range(3))
    perm = np.random.default_rng(5).permutation(N)
    a = attn(Q, K, V, 0.4, 0)
    b = attn(Q, K[:, :, perm, :], V[:, :, perm, :], 0.4, 0)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
    # permuting queries permutes output rows (no mask)
    c = attn(Q[:, :, perm, :], K, V, 0.4, 0)
    np.testing.assert_array_equal(c, a[:, :, perm, :])


def pin_logit_row_shift(attn):
    B, H, N, d = 1, 2, 27, 5
    Q, K, V = (rnd((B, H, N, d), 29, t) for t in range(3))
    c = rnd((d,), 31) * 3.0
    for mask in (0, 1):
        a = attn(Q, K, V, 0.9, mask)
        b = attn(Q, K + c, V, 0.9, mask)     # L_ij -> L_ij + scale * q_i.c : constant along each row
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


def pin_scaling_linearity_independence(attn):
    B, H, N, d = 2, 3, 21, 4
    Q, K, V = (rnd((B, H, N, d), 37, t) for t in range(3))
    V2 = rnd((B, H, N, d), 37, 5)
    for mask in (0, 1):
        a = attn(Q, K, V, 0.25, mask)
        np.testing.assert_array_equal(attn(2.0 * Q, K, V, 0.125, mask), a)   # power-of-two rescale is exact
        np.testing.assert_array_equal(attn(Q, 4.0 * K, V, 0.0625, mask), a)
        np.testing.assert_allclose(attn(Q, K, V + V2, 0.25, mask), a + attn(Q, K, V2, 0.25, mask), rtol=0, atol=1e-13)
        np.testing.assert_allclose(attn(Q, K, -3.0 * V, 0.25, mask), -3.0 * a, rtol=0, atol=1e-13)
        for b in range(B):
            for h in range(H):
                one = attn(Q[b:b + 1, h:h + 1], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], 0.25, mask)
                np.testing.assert_array_equal(one[0, 0], a[b, h])
    # scale really multiplies the logit: scale 0 gives uniform weights
    np.testing.assert_allclose(attn(Q, K, V, 0.0, 0), np.broadcast_to(V.mean(axis=2, keepdims=True), V.shape), rtol=0, atol=1e-14)


def pin_array_library(attn):
    """Float64 evaluation with an array library's matmul/exp as a second opinion, on rectangular N != d."""
    B, H, N, d = 2, 2, 45, 7
    Q, K, V = (rnd((B, H, N, d), 41, t) for t in range(3))
    for mask in (0, 1):
        L = np.einsum("bhik,bhjk->bhij", Q, K) * 0.3
        if mask:
            L = np.where(np.tril(np.ones((N, N), dtype=bool)), L, -np.inf)
        P = np.exp(L - L.max(axis=-1, keepdims=True))
        A = P / P.sum(axis=-1, keepdims=True)
        np.testing.assert_allclose(attn(Q, K, V, 0.3, mask), A @ V, rtol=0, atol=1e-13)


PINS = [pin_hand_example, pin_brute_force, pin_uniform_logits, pin_dominant_key, pin_constant_value_columns,
        pin_degenerate_rows, pin_permutation, pin_logit_row_shift, pin_scaling_linearity_independence, pin_array_library]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_pin(pin):
    pin(oracle_attn)


# ----------------------------------------------------------------------------- staged outputs
def test_softmax_rows_sum_to_one_and_mask_is_exact_zero():
    N, d = 203, 16
    Q, K = rnd((N, d), 43, 0, mult=2.0), rnd((N, d), 43, 1, mult=2.0)
    for mask in (0, 1):
        L, A = oracle.logits_softmax(Q, K, 0.35, mask)
        assert np.abs(A.sum(axis=1) - 1.0).max() <= 1e-12
        assert (A >= 0).all()
        want_L = (Q @ K.T) * 0.35
        vis = np.tril(np.ones((N, N), dtype=bool)) if mask else np.ones((N, N), dtype=bool)
        np.testing.assert_allclose(L[vis], want_L[vis], rtol=0, atol=1e-13)
        assert (A[~vis] == 0).all() and np.isneginf(L[~vis]).all()
        # monotone: larger logit, larger probability, within a row
        i = 57
        order = np.argsort(L[i][vis[i]])
        assert (np.diff(A[i][vis[i]][order]) >= 0).all()


def test_logits_are_query_dot_key_not_transposed():
    # N != d and asymmetric data: L[i, j] must be q_i . k_j
    Q = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    K = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    L, _ = oracle.logits_softmax(Q, K, 2.0, 0)
    np.testing.assert_array_equal(L, 2.0 * np.array([[1, 2, 3], [3, 4, 7], [5, 6, 11]], dtype=np.float64))


def test_row_subset_and_thread_count_do_not_change_results():
    w = synth.custom("t", 2, 3, 131, 8, seed=47)
    Q, K, V = synth.make_qkv(w)
    full1 = oracle.attention(Q, K, V, w.scale, 1, threads=1)
    full8 = oracle.attention(Q, K, V, w.scale, 1, threads=8)
    np.testing.assert_array_equal(full1, full8)
    rows = np.array([0, 130, 64, 63, 1, 77])
    sub = oracle.attention(Q, K, V, w.scale, 1, rows=rows, threads=3)
    np.testing.assert_array_equal(sub, full1[:, :, rows, :])


def test_bad_arguments_are_rejected():
    Q = np.zeros((1, 1, 4, 2))
    with pytest.raises(ValueError):
        oracle.attention(Q, Q, Q, 1.0, 2)
    with pytest.raises(ValueError):
        oracle.attention(Q, Q, Q, 1.0, 0, rows=np.array([4]))
    with pytest.raises(ValueError):
        oracle.attention(Q, Q[:, :, :3], Q, 1.0, 0)


def test_config0_against_array_library():
    """BERT-base-shaped workload, all rows: the oracle against a float64 matmul/exp evaluation."""
    w = synth.WORKLOADS["cfg0_bert_base_f32"]
    Q, K, V = (x.astype(np.float64) for x in synth.make_qkv(w))
    got = oracle.attention(Q, K, V, w.scale, w.mask)
    L = np.einsum("bhik,bhjk->bhij", Q, K) * w.scale
    P = np.exp(L - L.max(axis=-1, keepdims=True))
    want = (P / P.sum(axis=-1, keepdims=True)) @ V
    np.testing.assert_allclose(got, want, rtol=0, atol=5e-14)


# ----------------------------------------------------------------------------- the pins have teeth
def _np_attention(Q, K, V, scale, mask, *, strict_causal=False, axis=-1, use_scale=True, swap_kv=False,
                  no_max=False, transpose_logits=False, sum_not_mean=False, k_index_shift=0):
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    if swap_kv:
        K, V = V, K
    if k_index_shift:
        K = np.roll(K, k_index_shift, axis=2)
    L = np.einsum("bhik,bhjk->bhij", Q, K)
    if transpose_logits:
        L = np.swapaxes(L, -1, -2)
    if use_scale:
        L = L * scale
    N = L.shape[-1]
    if mask == 1:
        tri = np.tril(np.ones((N, N), dtype=bool), -1 if strict_causal else 0)
        if strict_causal:
            tri[0, 0] = True
        L = np.where(tri, L, -np.inf)
    if no_max:
        P = np.exp(L)
    else:
        P = np.exp(L - L.max(axis=-1, keepdims=True))
    P = np.where(np.isnan(P), 0.0, P)
    A = P if sum_not_mean else P / P.sum(axis=axis, keepdims=True)
    return A @ V


MUTANTS = {
    "causal_excludes_diagonal": dict(strict_causal=True),
    "softmax_over_queries": dict(axis=-2),
    "scale_dropped": dict(use_scale=False),
    "keys_and_values_swapped": dict(swap_kv=True),
    "no_max_subtraction": dict(no_max=True),
    "logits_transposed": dict(transpose_logits=True),
    "not_normalised": dict(sum_not_mean=True),
    "key_index_off_by_one": dict(k_index_shift=1),
}


def test_correct_numpy_version_passes_all_pins():
    for pin in PINS:
        pin(lambda Q, K, V, s, m: _np_attention(Q, K, V, s, m))


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    kw = MUTANTS[name]

    def mutant(Q, K, V, s, m):
        with np.errstate(all="ignore"):
            return _np_attention(Q, K, V, s, m, **kw)

    caught = []
    for pin in PINS:
        try:
            pin(mutant)
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the mistake '{name}'"


# ----------------------------------------------------------------------------- input generator
def test_generator_is_counter_based_and_distributed_as_stated():
    a = synth.tensor_f32((4, 1000), 3, synth.TENSOR_Q)
    b = synth.tensor_f32((4000,), 3, synth.TENSOR_Q)
    np.testing.assert_array_equal(a.reshape(-1), b)
    c = synth.tensor_f32((4000,), 3, synth.TENSOR_K)
    assert not np.array_equal(b, c)
    big = synth.tensor_f32((1 << 20,), 9, 0).astype(np.float64)
    assert abs(big.mean()) < 5e-3 and abs(big.std() - 1.0) < 5e-3
    assert abs(np.mean(big ** 4) - 3.0) < 0.05
    u = synth.tensor_f32((1 << 20,), 9, 2, "uniform").astype(np.float64)
    assert u.min() >= -1.0 and u.max() <= 1.0 and abs(u.mean()) < 5e-3 and abs(u.var() - 1.0 / 3.0) < 5e-3


def test_bf16_rounding_is_nearest_even_and_round_trips():
    x = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 3.140625, 0.0], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even (1.0); 1 + 3*2^-8 is a tie -> 1 + 2^-6 (even mantissa)
    got = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    np.testing.assert_array_equal(got, np.array([1.0, 1.0, 1.015625, -1.0, 3.140625, 0.0], dtype=np.float32))
    y = synth.tensor_f32((5000,), 1, 0)
    b = synth.f32_to_bf16_bits(y)
    back = synth.bf16_bits_to_f32(b)
    assert np.abs(back - y).max() <= np.abs(y).max() * 2.0 ** -8
    np.testing.assert_array_equal(synth.f32_to_bf16_bits(back), b)
    import torch
    t = torch.from_numpy(y).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(t, b)
