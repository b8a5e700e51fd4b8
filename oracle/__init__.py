"""ctypes front end of the CPU attention oracle (oracle/flat_oracle.cpp).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this; it is
for tests/, the smoke check and the benchmark's cpu_baseline leg.  It imports
nothing from the GPU package either.

`build()` compiles the C++ with g++; `attention()` and `logits_softmax()`
marshal numpy float64 arrays into it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flat_oracle.cpp")
_LIB = os.path.join(_HERE, "libflat_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle into oracle/libflat_oracle.so (rebuilds when the source is newer)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread",
                               "-ffp-contract=off", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        lib.flat_oracle_hw_threads.restype = ctypes.c_int
        lib.flat_oracle_attention.restype = ctypes.c_int
        lib.flat_oracle_attention.argtypes = [dp, dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                              ctypes.c_double, ctypes.c_int, ip, ctypes.c_int64, ctypes.c_int]
        lib.flat_oracle_attention_cross.restype = ctypes.c_int
        lib.flat_oracle_attention_cross.argtypes = [dp, dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                                    ctypes.c_int, ctypes.c_double, ctypes.c_int, ip, ip, ctypes.c_int64,
                                                    ctypes.c_int]
        lib.flat_oracle_attention_blocksparse.restype = ctypes.c_int
        lib.flat_oracle_attention_blocksparse.argtypes = [dp, dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                                          ctypes.c_double, ctypes.c_int64, ctypes.c_int64, ip, ip, ip,
                                                          ctypes.c_int64, ctypes.c_int]
        lib.flat_oracle_logits_softmax.restype = ctypes.c_int
        lib.flat_oracle_logits_softmax.argtypes = [dp, dp, ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                                   ip, ctypes.c_int64, dp, dp]
        _lib = lib
    return _lib


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def hw_threads() -> int:
    return int(_load().flat_oracle_hw_threads())


def attention(Q, K, V, scale: float, mask_kind: int = 0, rows=None, threads: int = 0) -> np.ndarray:
    """O = softmax_row(Q K^T * scale) V for [B,H,N,d] inputs, in float64.

    `rows` (1-D integer array) restricts the output to those query indices of
    every head; the result is [B,H,len(rows),d].  `scale` is used as given
    (pass the float32-rounded value that the GPU entry point receives).
    """
    lib = _load()
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    if Q.ndim != 4 or Q.shape != K.shape or Q.shape != V.shape:
        raise ValueError("Q, K, V must share a [B,H,N,d] shape")
    B, H, N, d = Q.shape
    if rows is None:
        rp, nr = None, N
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rp, nr = rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), rows.size
    O = np.empty((B, H, nr, d), dtype=np.float64)
    rc = lib.flat_oracle_attention(_dptr(Q), _dptr(K), _dptr(V), _dptr(O), B, H, N, d, float(scale), int(mask_kind),
                                   rp, nr, int(threads))
    if rc != 0:
        raise ValueError(f"flat_oracle_attention rejected its arguments (code {rc})")
    return O


def attention_cross(Q, K, V, scale: float, mask_kind: int = 0, kv_lens=None, rows=None, threads: int = 0) -> np.ndarray:
    """Attention of Q [B,H,Nq,d] over K, V [B,H,Nk,d] in float64 -> [B,H,len(rows) or Nq,d].

    Causal: the queries are the last Nq positions of the key sequence (needs Nk >= Nq).  `kv_lens` (B
    integers) limits batch entry b to its first kv_lens[b] keys.
    """
    lib = _load()
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    if Q.ndim != 4 or K.ndim != 4 or K.shape != V.shape or Q.shape[:2] != K.shape[:2] or Q.shape[3] != K.shape[3]:
        raise ValueError("Q must be [B,H,Nq,d] and K, V [B,H,Nk,d]")
    B, H, Nq, d = Q.shape
    Nk = K.shape[2]
    ip = ctypes.POINTER(ctypes.c_int64)
    lp = None
    if kv_lens is not None:
        kv_lens = np.ascontiguousarray(kv_lens, dtype=np.int64)
        if kv_lens.shape != (B,):
            raise ValueError("kv_lens must hold one count per batch entry")
        lp = kv_lens.ctypes.data_as(ip)
    if rows is None:
        rp, nr = None, Nq
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rp, nr = rows.ctypes.data_as(ip), rows.size
    O = np.empty((B, H, nr, d), dtype=np.float64)
    rc = lib.flat_oracle_attention_cross(_dptr(Q), _dptr(K), _dptr(V), _dptr(O), B, H, Nq, Nk, d, float(scale), int(mask_kind),
                                         lp, rp, nr, int(threads))
    if rc != 0:
        raise ValueError(f"flat_oracle_attention_cross rejected its arguments (code {rc})")
    return O


def attention_blocksparse(Q, K, V, scale: float, tile_offsets, tile_ids, block_rows: int = 256, block_keys: int = 64,
                          rows=None, threads: int = 0) -> np.ndarray:
    """Block-sparse attention in float64: query i sees key j iff tile j // block_keys is listed (CSR arrays
    `tile_offsets`, `tile_ids`) for row block i // block_rows of its (batch, head).  [B,H,N,d] -> [B,H,len(rows) or N,d]."""
    lib = _load()
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    if Q.ndim != 4 or Q.shape != K.shape or Q.shape != V.shape:
        raise ValueError("Q, K, V must share a [B,H,N,d] shape")
    B, H, N, d = Q.shape
    ip = ctypes.POINTER(ctypes.c_int64)
    offs = np.ascontiguousarray(tile_offsets, dtype=np.int64)
    ids = np.ascontiguousarray(tile_ids, dtype=np.int64)
    n_lists = B * H * ((N + block_rows - 1) // block_rows)
    if offs.shape != (n_lists + 1,) or ids.ndim != 1 or (offs[-1] != ids.size):
        raise ValueError("tile_offsets must have one entry per row block plus one and end at len(tile_ids)")
    if ids.size == 0:
        ids = np.zeros(1, dtype=np.int64)  # keeps the pointer valid; nothing is read
    if rows is None:
        rp, nr = None, N
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rp, nr = rows.ctypes.data_as(ip), rows.size
    O = np.empty((B, H, nr, d), dtype=np.float64)
    rc = lib.flat_oracle_attention_blocksparse(_dptr(Q), _dptr(K), _dptr(V), _dptr(O), B, H, N, d, float(scale),
                                               int(block_rows), int(block_keys), offs.ctypes.data_as(ip), ids.ctypes.data_as(ip),
                                               rp, nr, int(threads))
    if rc != 0:
        raise ValueError(f"flat_oracle_attention_blocksparse rejected its arguments (code {rc})")
    return O


def logits_softmax(Q, K, scale: float, mask_kind: int = 0, rows=None):
    """(L, A) of one head: Q, K are [N,d]; returns two [len(rows), N] float64 arrays."""
    lib = _load()
    Q, K = _f64(Q), _f64(K)
    N, d = Q.shape
    rows = np.arange(N, dtype=np.int64) if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    L = np.empty((rows.size, N), dtype=np.float64)
    A = np.empty((rows.size, N), dtype=np.float64)
    rc = lib.flat_oracle_logits_softmax(_dptr(Q), _dptr(K), N, d, float(scale), int(mask_kind),
                                        rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), rows.size, _dptr(L), _dptr(A))
    if rc != 0:
        raise ValueError(f"flat_oracle_logits_softmax rejected its arguments (code {rc})")
    return L, A
