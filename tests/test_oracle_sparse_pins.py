"""Pins for the oracle's block-sparse attention (oracle.attention_blocksparse).

The paper prunes the N x N matrix randomly and does not define a block pattern, so the pins are reductions:
  * every tile listed: plain attention (oracle.attention);
  * the first t tiles listed: attention over K, V truncated to t tiles;
  * any list: the test gathers the listed keys itself and calls the pinned cross-length attention on them, row
    block by row block;
  * brute force with an explicit visibility test per (query, key) pair.
The pins take the function under test as an argument and are run against planted mistakes too.
"""
import numpy as np
import pytest

import oracle
from paper_2107_06419_amd import synth


def rnd(shape, seed, tid=0):
    return synth.tensor_f32(shape, seed, tid, "normal", 1.0).astype(np.float64)


def full_pattern(n_lists, n_kt):
    return np.arange(n_lists + 1, dtype=np.int64) * n_kt, np.tile(np.arange(n_kt, dtype=np.int64), n_lists)


def pin_all_tiles_is_dense(sparse):
    B, H, N, d, br, bk = 2, 2, 37, 3, 8, 4
    Q, K, V = (rnd((B, H, N, d), 5, t) for t in range(3))
    offs, ids = full_pattern(B * H * 5, 10)
    np.testing.assert_allclose(sparse(Q, K, V, 0.6, offs, ids, br, bk), oracle.attention(Q, K, V, 0.6, 0), rtol=0, atol=1e-14)


def pin_prefix_of_tiles_is_truncation(sparse):
    B, H, N, d, br, bk = 1, 2, 30, 4, 16, 4
    Q, K, V = (rnd((B, H, N, d), 9, t) for t in range(3))
    n_lists, t = B * H * 2, 5
    offs = np.arange(n_lists + 1, dtype=np.int64) * t
    ids = np.tile(np.arange(t, dtype=np.int64), n_lists)
    want = oracle.attention_cross(Q, K[:, :, :t * bk], V[:, :, :t * bk], 0.9, 0)
    np.testing.assert_allclose(sparse(Q, K, V, 0.9, offs, ids, br, bk), want, rtol=0, atol=1e-14)


def pin_gathered_keys(sparse):
    B, H, N, d, br, bk = 2, 2, 45, 3, 8, 6            # ragged: last row block has 5 rows, last key tile 3 keys
    Q, K, V = (rnd((B, H, N, d), 13, t) for t in range(3))
    n_rb, n_kt = 6, 8
    offs, ids = synth.random_block_pattern(B * H * n_rb, n_kt, 0.4, seed=77)
    got = sparse(Q, K, V, 0.5, offs, ids, br, bk)
    for bh in range(B * H):
        b, h = divmod(bh, H)
        for rb in range(n_rb):
            lst = ids[offs[bh * n_rb + rb]:offs[bh * n_rb + rb + 1]]
            keys = np.concatenate([np.arange(t * bk, min((t + 1) * bk, N)) for t in lst])
            r0, r1 = rb * br, min((rb + 1) * br, N)
            want = oracle.attention_cross(Q[b:b + 1, h:h + 1, r0:r1], K[b:b + 1, h:h + 1, keys], V[b:b + 1, h:h + 1, keys], 0.5, 0)
            np.testing.assert_allclose(got[b:b + 1, h:h + 1, r0:r1], want, rtol=0, atol=1e-14)


def _brute(Q, K, V, scale, offs, ids, br, bk):
    B, H, N, d = Q.shape
    n_rb = -(-N // br)
    ld = np.longdouble
    O = np.zeros((B, H, N, d))
    for b in range(B):
        for h in range(H):
            for i in range(N):
                r = (b * H + h) * n_rb + i // br
                listed = set(int(t) for t in ids[offs[r]:offs[r + 1]])
                w = []
                for j in range(N):
                    lij = sum(ld(Q[b, h, i, k]) * ld(K[b, h, j, k]) for k in range(d))
                    w.append(np.exp(lij * ld(scale)) if (j // bk) in listed else ld(0))
                den = sum(w)
                if den == 0:
                    continue
                for c in range(d):
                    O[b, h, i, c] = float(sum(w[j] * ld(V[b, h, j, c]) for j in range(N)) / den)
    return O


def pin_brute_force(sparse):
    for seed, (B, H, N, d, br, bk) in enumerate([(1, 1, 5, 2, 2, 2), (2, 1, 9, 2, 4, 3), (1, 2, 8, 3, 8, 2), (1, 1, 7, 1, 3, 7)]):
        Q, K, V = (rnd((B, H, N, d), 20 + seed, t) for t in range(3))
        offs, ids = synth.random_block_pattern(B * H * -(-N // br), -(-N // bk), 0.5, seed=seed, at_least_one=(seed % 2 == 0))
        np.testing.assert_allclose(sparse(Q, K, V, 0.8, offs, ids, br, bk), _brute(Q, K, V, 0.8, offs, ids, br, bk), rtol=0, atol=1e-13)


def pin_empty_list_gives_zero_rows(sparse):
    B, H, N, d, br, bk = 1, 1, 8, 2, 4, 4
    Q, K, V = (rnd((B, H, N, d), 31, t) for t in range(3))
    offs, ids = np.array([0, 0, 1]), np.array([1])
    got = sparse(Q, K, V, 1.0, offs, ids, br, bk)
    assert (got[0, 0, :4] == 0).all()
    np.testing.assert_allclose(got[0, 0, 4:], oracle.attention_cross(Q[:, :, 4:], K[:, :, 4:], V[:, :, 4:], 1.0, 0)[0, 0], rtol=0, atol=1e-14)


PINS = [pin_all_tiles_is_dense, pin_prefix_of_tiles_is_truncation, pin_gathered_keys, pin_brute_force, pin_empty_list_gives_zero_rows]


def oracle_sparse(Q, K, V, scale, offs, ids, br, bk):
    return oracle.attention_blocksparse(Q, K, V, scale, offs, ids, br, bk)


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_sparse_oracle_pin(pin):
    pin(oracle_sparse)


def _np_sparse(Q, K, V, scale, offs, ids, br, bk, *, swap_blocks=False, per_head_lists=True, clip=True, shift_list=0):
    """Array-library version with switches that plant plausible mistakes."""
    B, H, N, d = Q.shape
    if swap_blocks:
        br, bk = bk, br
    n_rb = -(-N // br)
    L = np.einsum("bhik,bhjk->bhij", Q, K) * scale
    vis = np.zeros((B, H, N, N), dtype=bool)
    for b in range(B):
        for h in range(H):
            for i in range(N):
                r = ((b * H + h) if per_head_lists else 0) * n_rb + i // br + shift_list
                r = min(r, len(offs) - 2)
                for t in ids[offs[r]:offs[r + 1]]:
                    hi = (t + 1) * bk if clip else (t + 1) * bk + 1
                    vis[b, h, i, t * bk:min(hi, N)] = True
    out = np.zeros(Q.shape)
    with np.errstate(all="ignore"):
        Lm = np.where(vis, L, -np.inf)
        P = np.exp(Lm - np.nanmax(np.where(vis, L, np.nan), axis=-1, keepdims=True, initial=-np.inf, where=vis))
        Z = P.sum(axis=-1, keepdims=True)
        P = np.where(Z > 0, P / np.where(Z > 0, Z, 1), 0.0)
    return np.einsum("bhij,bhjc->bhic", P, V)


def test_array_library_version_passes_all_pins():
    for pin in PINS:
        pin(lambda *a: _np_sparse(*a))


MUTANTS = {
    "row and key block sizes swapped": dict(swap_blocks=True),
    "one list shared by all heads": dict(per_head_lists=False),
    "a tile reaches one key into the next": dict(clip=False),
    "lists shifted by one row block": dict(shift_list=1),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    def mutant(*a):
        return _np_sparse(*a, **MUTANTS[name])
    failed = 0
    for pin in PINS:
        try:
            pin(mutant)
        except (AssertionError, IndexError, ValueError):
            failed += 1
    assert failed >= 1, f"no pin notices: {name}"


def test_bad_lists_are_rejected():
    Q = rnd((1, 1, 8, 2), 1, 0)
    for offs, ids in (([0, 1, 3], [0, 1, 1]), ([0, 1, 2], [0, 2]), ([0, 2, 1], [0, 1]), ([1, 1, 1], [0])):
        with pytest.raises(ValueError):
            oracle.attention_blocksparse(Q, Q, Q, 1.0, np.array(offs), np.array(ids), 4, 4)
    with pytest.raises(ValueError):
        oracle.attention_blocksparse(Q, Q, Q, 1.0, np.array([0, 1]), np.array([0]), 4, 4)   # one offset too few
