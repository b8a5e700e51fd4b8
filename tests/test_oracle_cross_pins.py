"""Pins for the oracle's attention over Nq queries and Nk keys (oracle.attention_cross).

The paper does not define these cases, so the pins are reductions to what is already pinned and brute force:
  * Nq = Nk without key counts is plain self-attention (oracle.attention, pinned in test_oracle_pins.py);
  * causal: the queries are the last Nq positions, so the result is the last Nq rows of causal self-attention
    over all Nk positions (whatever the earlier queries are);
  * key counts: batch entry b behaves as if K and V ended after kv_lens[b] rows, whatever the padding holds;
  * per-element brute force with the visibility written as an explicit test per (query, key) pair.
Every pin takes the function under test as an argument and is also run against planted mistakes.
"""
import numpy as np
import pytest

import oracle
from paper_2107_06419_amd import synth


def rnd(shape, seed, tid=0):
    return synth.tensor_f32(shape, seed, tid, "normal", 1.0).astype(np.float64)


def pin_reduces_to_self_attention(cross):
    Q, K, V = (rnd((2, 3, 17, 4), 31, t) for t in range(3))
    for mask in (0, 1):
        np.testing.assert_allclose(cross(Q, K, V, 0.6, mask, None), oracle.attention(Q, K, V, 0.6, mask), rtol=0, atol=1e-14)
    full = np.array([17, 17])
    np.testing.assert_allclose(cross(Q, K, V, 0.6, 1, full), oracle.attention(Q, K, V, 0.6, 1), rtol=0, atol=1e-14)


def pin_tail_of_causal_self_attention(cross):
    B, H, Nk, d = 2, 2, 23, 5
    Qfull, K, V = (rnd((B, H, Nk, d), 37, t) for t in range(3))
    ref = oracle.attention(Qfull, K, V, 0.45, 1)
    for Nq in (1, 7, 22, 23):
        got = cross(Qfull[:, :, Nk - Nq:, :], K, V, 0.45, 1, None)
        np.testing.assert_allclose(got, ref[:, :, Nk - Nq:, :], rtol=0, atol=1e-14)
    # without a mask every query sees every key, wherever it sits
    ref = oracle.attention(Qfull, K, V, 0.45, 0)
    got = cross(Qfull[:, :, 5:9, :], K, V, 0.45, 0, None)
    np.testing.assert_allclose(got, ref[:, :, 5:9, :], rtol=0, atol=1e-14)


def pin_padding_equals_truncation(cross):
    B, H, Nq, Nk, d = 3, 2, 6, 19, 4
    Q = rnd((B, H, Nq, d), 41, 0)
    K, V = (rnd((B, H, Nk, d), 41, t) for t in (1, 2))
    lens = np.array([19, 1, 8])
    Kp, Vp = K.copy(), V.copy()
    for b in range(B):  # poison the padding: it must not matter
        Kp[b, :, lens[b]:, :] = 1e6
        Vp[b, :, lens[b]:, :] = -1e6
    got = cross(Q, Kp, Vp, 0.8, 0, lens)
    for b in range(B):
        want = cross(Q[b:b + 1], K[b:b + 1, :, :lens[b]], V[b:b + 1, :, :lens[b]], 0.8, 0, None)
        np.testing.assert_allclose(got[b:b + 1], want, rtol=0, atol=1e-14)
    # with the causal mask the alignment still refers to Nk: query i sees keys <= i + Nk - Nq that are below the count
    got = cross(Q, Kp, Vp, 0.8, 1, lens)
    off = Nk - Nq
    for b in range(B):
        for i in range(Nq):
            n = min(lens[b], i + off + 1)
            want = cross(Q[b:b + 1, :, i:i + 1], K[b:b + 1, :, :n], V[b:b + 1, :, :n], 0.8, 0, None)
            np.testing.assert_allclose(got[b:b + 1, :, i:i + 1], want, rtol=0, atol=1e-14)


def _brute(Q, K, V, scale, mask, lens):
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    ld = np.longdouble
    O = np.zeros((B, H, Nq, d))
    for b in range(B):
        for h in range(H):
            for i in range(Nq):
                w = []
                for j in range(Nk):
                    visible = (lens is None or j < lens[b]) and (mask == 0 or j - (Nk - Nq) <= i)
                    lij = sum(ld(Q[b, h, i, k]) * ld(K[b, h, j, k]) for k in range(d))
                    w.append(np.exp(lij * ld(scale)) if visible else ld(0))
                den = sum(w)
                for c in range(d):
                    O[b, h, i, c] = float(sum(w[j] * ld(V[b, h, j, c]) for j in range(Nk)) / den)
    return O


def pin_brute_force(cross):
    cases = [(1, 1, 1, 1, 1, None), (1, 2, 3, 7, 2, None), (2, 1, 4, 4, 3, [2, 4]), (2, 2, 2, 9, 2, [9, 3]), (1, 1, 5, 6, 1, [1])]
    for seed, (B, H, Nq, Nk, d, lens) in enumerate(cases):
        Q = rnd((B, H, Nq, d), 50 + seed, 0)
        K, V = (rnd((B, H, Nk, d), 50 + seed, t) for t in (1, 2))
        lens = None if lens is None else np.array(lens)
        for mask in (0, 1):
            np.testing.assert_allclose(cross(Q, K, V, 0.7, mask, lens), _brute(Q, K, V, 0.7, mask, lens), rtol=0, atol=1e-13)


def pin_uniform_logits(cross):
    B, H, Nq, Nk, d = 1, 2, 5, 12, 3
    Q = rnd((B, H, Nq, d), 61, 0)
    V = rnd((B, H, Nk, d), 61, 2)
    K = np.zeros((B, H, Nk, d))
    got = cross(Q, K, V, 1.0, 1, None)
    for i in range(Nq):  # mean of the keys this query sees: positions 0 .. i + 7
        np.testing.assert_allclose(got[:, :, i], V[:, :, :i + 8].mean(axis=2), rtol=0, atol=1e-14)
    got = cross(Q, K, V, 1.0, 0, np.array([4]))
    np.testing.assert_allclose(got, np.broadcast_to(V[:, :, :4].mean(axis=2, keepdims=True), got.shape), rtol=0, atol=1e-14)


PINS = [pin_reduces_to_self_attention, pin_tail_of_causal_self_attention, pin_padding_equals_truncation, pin_brute_force,
        pin_uniform_logits]


def oracle_cross(Q, K, V, scale, mask, lens):
    return oracle.attention_cross(Q, K, V, scale, mask, kv_lens=lens)


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_cross_oracle_pin(pin):
    pin(oracle_cross)


def _np_cross(Q, K, V, scale, mask, lens, *, align="end", ignore_lens=False, lens_after_mask=False, strict=False):
    """Array-library version with switches that plant the plausible mistakes."""
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    L = np.einsum("bhik,bhjk->bhij", Q, K) * scale
    i = np.arange(Nq)[:, None]
    j = np.arange(Nk)[None, :]
    vis = np.ones((B, 1, Nq, Nk), dtype=bool)
    if mask == 1:
        off = Nk - Nq if align == "end" else 0
        vis = vis & ((j < i + off) if strict else (j <= i + off))[None, None]
    if lens is not None and not ignore_lens:
        lim = np.asarray(lens)[:, None, None, None]
        if lens_after_mask and mask == 1:
            lim = lim + 1
        vis = vis & (j[None, None] < lim)
    L = np.where(vis, L, -np.inf)
    L = L - L.max(axis=-1, keepdims=True)
    P = np.exp(L)
    P = P / P.sum(axis=-1, keepdims=True)
    return np.einsum("bhij,bhjc->bhic", P, V)


def test_array_library_version_passes_all_pins_and_agrees():
    for pin in PINS:
        pin(lambda *a: _np_cross(*a))
    Q = rnd((2, 2, 9, 8), 71, 0)
    K, V = (rnd((2, 2, 30, 8), 71, t) for t in (1, 2))
    for mask in (0, 1):
        for lens in (None, np.array([30, 11])):
            np.testing.assert_allclose(oracle_cross(Q, K, V, 0.35, mask, lens), _np_cross(Q, K, V, 0.35, mask, lens), rtol=0, atol=1e-13)


MUTANTS = {
    "causal aligned to the first key instead of the last": dict(align="start"),
    "key counts ignored": dict(ignore_lens=True),
    "key count off by one under the causal mask": dict(lens_after_mask=True),
    "diagonal excluded": dict(strict=True),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    def mutant(*a):
        return _np_cross(*a, **MUTANTS[name])
    failed = 0
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin(mutant)
        except AssertionError:
            failed += 1
    assert failed >= 1, f"no pin notices: {name}"


def test_bad_arguments_are_rejected():
    Q = rnd((1, 1, 4, 2), 1, 0)
    K = rnd((1, 1, 3, 2), 1, 1)
    with pytest.raises(ValueError):
        oracle.attention_cross(Q, K, K, 1.0, 1)                      # causal needs Nk >= Nq
    with pytest.raises(ValueError):
        oracle.attention_cross(Q, K, K, 1.0, 0, kv_lens=np.array([0]))
    with pytest.raises(ValueError):
        oracle.attention_cross(Q, K, K, 1.0, 0, kv_lens=np.array([4]))
    with pytest.raises(ValueError):
        oracle.attention_cross(Q, K, K, 1.0, 0, rows=np.array([4]))
    assert oracle.attention_cross(Q, K, K, 1.0, 0, rows=np.array([3, 0])).shape == (1, 1, 2, 2)
