"""ctypes binding of include/flat_attn.h.  Same names as the C entry points; argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device buffers: the binding passes
`data_ptr()` and the current HIP stream to the library and returns the C status code turned into
an exception.  Nothing here computes.
"""
from __future__ import annotations

import ctypes
import os

FLAT_MASK_NONE = 0
FLAT_MASK_CAUSAL = 1
FLAT_DTYPE_BF16 = 0

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libflat_attn.so")
_PROBE_LIB_PATH = os.path.join(_HERE, "libflat_attn_probe.so")
_lib = None
_probe_lib = None


class FlatAttnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{message} (status {status})")
        self.status = status


class FlatTileShape(ctypes.Structure):
    """flat_tile_shape of the header, field for field."""
    _fields_ = [(n, ctypes.c_int) for n in ("d", "rows_per_workgroup", "keys_per_tile", "wavefronts", "rows_per_wavefront",
                                            "lds_stages", "lds_bytes")]

    def as_dict(self) -> dict:
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


def library_path() -> str:
    return _LIB_PATH


def probe_library_path() -> str:
    return _PROBE_LIB_PATH


def load_probe_library():
    """Load libflat_attn_probe.so (the measurement aids of include/flat_attn_probe.h); raises if it has not been built."""
    global _probe_lib
    if _probe_lib is not None:
        return _probe_lib
    if not os.path.exists(_PROBE_LIB_PATH):
        raise FileNotFoundError(
            f"{_PROBE_LIB_PATH} is missing: build it with `python -m paper_2107_06419_amd.build` (needs hipcc)")
    try:
        import torch  # noqa: F401  (same HIP runtime as the tensors)
    except ImportError:
        pass
    lib = ctypes.CDLL(_PROBE_LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.flat_attn_mfma_probe_sink_bytes.restype = sz
    lib.flat_attn_mfma_probe_sink_bytes.argtypes = []
    lib.flat_attn_mfma_probe_flops.restype = ctypes.c_double
    lib.flat_attn_mfma_probe_flops.argtypes = [i]
    lib.flat_attn_mfma_probe.restype = i
    lib.flat_attn_mfma_probe.argtypes = [vp, sz, i, i, vp]
    lib.flat_attn_mix_probe_sink_bytes.restype = sz
    lib.flat_attn_mix_probe_sink_bytes.argtypes = []
    lib.flat_attn_mix_probe_src_bytes.restype = sz
    lib.flat_attn_mix_probe_src_bytes.argtypes = []
    lib.flat_attn_mix_probe_flops.restype = ctypes.c_double
    lib.flat_attn_mix_probe_flops.argtypes = [i]
    lib.flat_attn_mix_probe.restype = i
    lib.flat_attn_mix_probe.argtypes = [vp, sz, vp, sz, i, i, vp]
    _probe_lib = lib
    return lib


def load_library():
    """Load libflat_attn.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2107_06419_amd.build` (needs hipcc)")
    # The device pointers and streams this binding hands over come from torch's HIP runtime.  Importing torch
    # first makes the dynamic linker bind the library to that same runtime instead of loading a second one.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i, f, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.flat_attn_fwd.restype = i
    lib.flat_attn_fwd.argtypes = [vp, vp, vp, vp, i, i, i, i, f, i, vp]
    lib.flat_attn_fwd_cross.restype = i
    lib.flat_attn_fwd_cross.argtypes = [vp, vp, vp, vp, i, i, i, i, i, f, i, vp, vp]
    lib.flat_attn_fwd_splitkv_splits.restype = i
    lib.flat_attn_fwd_splitkv_splits.argtypes = [i, i, i, i, i, i]
    lib.flat_attn_fwd_splitkv_workspace_bytes.restype = sz
    lib.flat_attn_fwd_splitkv_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.flat_attn_fwd_splitkv.restype = i
    lib.flat_attn_fwd_splitkv.argtypes = [vp, vp, vp, vp, i, i, i, i, i, f, i, vp, i, vp, sz, vp]
    lib.flat_attn_fwd_splitkv_static.restype = i
    lib.flat_attn_fwd_splitkv_static.argtypes = [vp, vp, vp, vp, i, i, i, i, i, f, i, vp, i, vp]
    lib.flat_attn_fwd_blocksparse.restype = i
    lib.flat_attn_fwd_blocksparse.argtypes = [vp, vp, vp, vp, i, i, i, i, f, vp, vp, i, vp]
    lib.flat_attn_fwd_f32.restype = i
    lib.flat_attn_fwd_f32.argtypes = [vp, vp, vp, vp, i, i, i, i, f, i, vp]
    lib.flat_attn_unfused_workspace_bytes.restype = sz
    lib.flat_attn_unfused_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.flat_attn_unfused.restype = i
    lib.flat_attn_unfused.argtypes = [vp, vp, vp, vp, i, i, i, i, f, i, vp, sz, i, vp]
    lib.flat_attn_tile_shape_count.restype = i
    lib.flat_attn_tile_shape_count.argtypes = [i]
    lib.flat_attn_tile_shape_get.restype = i
    lib.flat_attn_tile_shape_get.argtypes = [i, i, ctypes.POINTER(FlatTileShape)]
    lib.flat_attn_tile_shape_occupancy.restype = i
    lib.flat_attn_tile_shape_occupancy.argtypes = [i, i]
    lib.flat_attn_tile_shape_default.restype = i
    lib.flat_attn_tile_shape_default.argtypes = [i, i, i, i, i]
    lib.flat_attn_fwd_tile.restype = i
    lib.flat_attn_fwd_tile.argtypes = [vp, vp, vp, vp, i, i, i, i, f, i, i, vp]
    lib.flat_attn_status_string.restype = ctypes.c_char_p
    lib.flat_attn_status_string.argtypes = [i]
    lib.flat_attn_version.restype = i
    lib.flat_attn_version.argtypes = []
    _lib = lib
    return lib


def flat_attn_status_string(status: int) -> str:
    return load_library().flat_attn_status_string(int(status)).decode()


def flat_attn_version() -> int:
    return int(load_library().flat_attn_version())


def _check(status: int) -> None:
    if status != 0:
        raise FlatAttnError(status, flat_attn_status_string(status))


def _stream_handle(stream) -> int:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_args(dtype, *tensors):
    shape = tensors[0].shape
    if len(shape) != 4:
        raise ValueError("expected [B, H, N, d] tensors")
    for t in tensors:
        if not t.is_cuda:
            raise ValueError("tensors must live on the GPU")
        if t.dtype != dtype:
            raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
        if t.shape != shape or not t.is_contiguous():
            raise ValueError("tensors must be contiguous and share one [B, H, N, d] shape")
    return tuple(int(s) for s in shape)


def flat_attn_fwd(Q, K, V, O, scale: float, mask_kind: int = FLAT_MASK_NONE, stream=None) -> None:
    """Fused attention, bf16 [B,H,N,d] device tensors; O is overwritten. Enqueues on `stream`."""
    import torch
    B, H, N, d = _dev_args(torch.bfloat16, Q, K, V, O)
    _check(load_library().flat_attn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                        float(scale), int(mask_kind), _stream_handle(stream)))


def flat_attn_fwd_cross(Q, K, V, O, scale: float, mask_kind: int = FLAT_MASK_NONE, kv_lens=None, stream=None) -> None:
    """Fused attention with Nq queries and Nk keys: Q, O bf16 [B,H,Nq,d], K, V bf16 [B,H,Nk,d] device tensors;
    kv_lens: optional int32 device tensor of B key counts (padding beyond them is ignored)."""
    import torch
    B, H, Nq, d = _dev_args(torch.bfloat16, Q, O)
    Bk, Hk, Nk, dk = _dev_args(torch.bfloat16, K, V)
    if (Bk, Hk, dk) != (B, H, d):
        raise ValueError("K, V must share batch, heads and head size with Q")
    lens_ptr = None
    if kv_lens is not None:
        if not kv_lens.is_cuda or kv_lens.dtype != torch.int32 or not kv_lens.is_contiguous() or kv_lens.numel() != B:
            raise ValueError("kv_lens must be a contiguous int32 GPU tensor with one entry per batch")
        lens_ptr = kv_lens.data_ptr()
    _check(load_library().flat_attn_fwd_cross(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, Nq, Nk, d,
                                              float(scale), int(mask_kind), lens_ptr, _stream_handle(stream)))


def flat_attn_fwd_splitkv_splits(B: int, H: int, Nq: int, Nk: int, d: int, n_splits: int = 0) -> int:
    """Number of splits a flat_attn_fwd_splitkv call with these arguments uses (n_splits <= 0: the library's choice)."""
    n = int(load_library().flat_attn_fwd_splitkv_splits(int(B), int(H), int(Nq), int(Nk), int(d), int(n_splits)))
    if n < 0:
        _check(n)
    return n


def flat_attn_fwd_splitkv_workspace_bytes(B: int, H: int, Nq: int, Nk: int, d: int, n_splits: int = 0) -> int:
    return int(load_library().flat_attn_fwd_splitkv_workspace_bytes(int(B), int(H), int(Nq), int(Nk), int(d), int(n_splits)))


def _cross_args(Q, K, V, O, kv_lens):
    import torch
    B, H, Nq, d = _dev_args(torch.bfloat16, Q, O)
    Bk, Hk, Nk, dk = _dev_args(torch.bfloat16, K, V)
    if (Bk, Hk, dk) != (B, H, d):
        raise ValueError("K, V must share batch, heads and head size with Q")
    lens_ptr = None
    if kv_lens is not None:
        if not kv_lens.is_cuda or kv_lens.dtype != torch.int32 or not kv_lens.is_contiguous() or kv_lens.numel() != B:
            raise ValueError("kv_lens must be a contiguous int32 GPU tensor with one entry per batch")
        lens_ptr = kv_lens.data_ptr()
    return B, H, Nq, Nk, d, lens_ptr


def flat_attn_fwd_splitkv(Q, K, V, O, scale: float, mask_kind: int, kv_lens, n_splits: int, workspace, stream=None) -> None:
    """flat_attn_fwd_cross with the keys of every row block divided over n_splits workgroups (<= 0: library's choice);
    `workspace` is a device tensor of at least flat_attn_fwd_splitkv_workspace_bytes() bytes."""
    B, H, Nq, Nk, d, lens_ptr = _cross_args(Q, K, V, O, kv_lens)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    _check(load_library().flat_attn_fwd_splitkv(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, Nq, Nk, d,
                                                float(scale), int(mask_kind), lens_ptr, int(n_splits), workspace.data_ptr(),
                                                workspace.numel() * workspace.element_size(), _stream_handle(stream)))


FLAT_SPLITKV_STATIC_BYTES = 64 << 20


def flat_attn_fwd_splitkv_static(Q, K, V, O, scale: float, mask_kind: int, kv_lens=None, n_splits: int = 0, stream=None) -> None:
    """flat_attn_fwd_splitkv out of the library's built-in scratch buffer (FLAT_SPLITKV_STATIC_BYTES): allocates nothing."""
    B, H, Nq, Nk, d, lens_ptr = _cross_args(Q, K, V, O, kv_lens)
    _check(load_library().flat_attn_fwd_splitkv_static(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, Nq, Nk, d,
                                                       float(scale), int(mask_kind), lens_ptr, int(n_splits), _stream_handle(stream)))


FLAT_SPARSE_BLOCK_ROWS = 256
FLAT_SPARSE_BLOCK_KEYS = 64


def flat_attn_fwd_blocksparse(Q, K, V, O, scale: float, tile_offsets, tile_ids, stream=None) -> None:
    """Block-sparse fused attention: int32 device tensors `tile_offsets` (B*H*ceil(N/256) + 1) and `tile_ids` list,
    per block of 256 query rows, the 64-key tiles it sees (CSR, ids ascending)."""
    import torch
    B, H, N, d = _dev_args(torch.bfloat16, Q, K, V, O)
    for t in (tile_offsets, tile_ids):
        if not t.is_cuda or t.dtype != torch.int32 or not t.is_contiguous():
            raise ValueError("tile_offsets and tile_ids must be contiguous int32 GPU tensors")
    n_row_blocks = B * H * ((N + FLAT_SPARSE_BLOCK_ROWS - 1) // FLAT_SPARSE_BLOCK_ROWS)
    if tile_offsets.numel() != n_row_blocks + 1:
        raise ValueError(f"tile_offsets must have {n_row_blocks + 1} entries")
    _check(load_library().flat_attn_fwd_blocksparse(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                                    float(scale), tile_offsets.data_ptr(), tile_ids.data_ptr(),
                                                    int(tile_ids.numel()), _stream_handle(stream)))


def flat_attn_fwd_f32(Q, K, V, O, scale: float, mask_kind: int = FLAT_MASK_NONE, stream=None) -> None:
    """Fused attention in fp32, float32 [B,H,N,d] device tensors."""
    import torch
    B, H, N, d = _dev_args(torch.float32, Q, K, V, O)
    _check(load_library().flat_attn_fwd_f32(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                            float(scale), int(mask_kind), _stream_handle(stream)))


def flat_attn_unfused_workspace_bytes(B: int, H: int, N: int, d: int, dtype: int = FLAT_DTYPE_BF16) -> int:
    return int(load_library().flat_attn_unfused_workspace_bytes(int(B), int(H), int(N), int(d), int(dtype)))


def flat_attn_unfused(Q, K, V, O, scale: float, mask_kind: int, workspace, stream=None) -> None:
    """Unfused baseline; `workspace` is a device tensor of at least flat_attn_unfused_workspace_bytes() bytes."""
    import torch
    B, H, N, d = _dev_args(torch.bfloat16, Q, K, V, O)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().flat_attn_unfused(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                            float(scale), int(mask_kind), workspace.data_ptr(), nbytes,
                                            FLAT_DTYPE_BF16, _stream_handle(stream)))


def flat_attn_tile_shape_count(d: int) -> int:
    return int(load_library().flat_attn_tile_shape_count(int(d)))


def flat_attn_tile_shape_get(d: int, index: int) -> FlatTileShape:
    out = FlatTileShape()
    _check(load_library().flat_attn_tile_shape_get(int(d), int(index), ctypes.byref(out)))
    return out


def flat_attn_tile_shape_occupancy(d: int, index: int) -> int:
    """Workgroups of the shape resident per compute unit on the current device (needs a GPU)."""
    n = int(load_library().flat_attn_tile_shape_occupancy(int(d), int(index)))
    if n < 0:
        _check(n)
    return n


def flat_attn_tile_shape_default(B: int, H: int, Nq: int, d: int, mask_kind: int = FLAT_MASK_NONE) -> int:
    """Index of the tile shape flat_attn_fwd / flat_attn_fwd_cross take for this problem (host arithmetic only)."""
    n = int(load_library().flat_attn_tile_shape_default(int(B), int(H), int(Nq), int(d), int(mask_kind)))
    if n < 0:
        _check(n)
    return n


def flat_attn_fwd_tile(Q, K, V, O, scale: float, mask_kind: int, tile_shape: int, stream=None) -> None:
    """flat_attn_fwd with tile shape `tile_shape` of the library's table instead of the default (index 0)."""
    import torch
    B, H, N, d = _dev_args(torch.bfloat16, Q, K, V, O)
    _check(load_library().flat_attn_fwd_tile(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), B, H, N, d,
                                             float(scale), int(mask_kind), int(tile_shape), _stream_handle(stream)))


def flat_attn_mfma_probe_sink_bytes() -> int:
    return int(load_probe_library().flat_attn_mfma_probe_sink_bytes())


def flat_attn_mfma_probe_flops(iters: int) -> float:
    return float(load_probe_library().flat_attn_mfma_probe_flops(int(iters)))


def flat_attn_mfma_probe(sink, iters: int, random_operands: bool, stream=None) -> None:
    """MFMA-only throughput probe; `sink` is a device tensor of at least flat_attn_mfma_probe_sink_bytes() bytes."""
    if not sink.is_cuda or not sink.is_contiguous():
        raise ValueError("sink must be a contiguous GPU tensor")
    _check(load_probe_library().flat_attn_mfma_probe(sink.data_ptr(), sink.numel() * sink.element_size(), int(iters),
                                               1 if random_operands else 0, _stream_handle(stream)))


def flat_attn_mix_probe_sink_bytes() -> int:
    return int(load_probe_library().flat_attn_mix_probe_sink_bytes())


def flat_attn_mix_probe_src_bytes() -> int:
    return int(load_probe_library().flat_attn_mix_probe_src_bytes())


def flat_attn_mix_probe_flops(iters: int) -> float:
    return float(load_probe_library().flat_attn_mix_probe_flops(int(iters)))


def flat_attn_mix_probe(sink, src, level: int, iters: int, stream=None) -> None:
    """Instruction-mix probe of the fused kernel's step; `sink` / `src` are device tensors of at least
    flat_attn_mix_probe_sink_bytes() / flat_attn_mix_probe_src_bytes() bytes."""
    if not sink.is_cuda or not sink.is_contiguous() or not src.is_cuda or not src.is_contiguous():
        raise ValueError("sink and src must be contiguous GPU tensors")
    _check(load_probe_library().flat_attn_mix_probe(sink.data_ptr(), sink.numel() * sink.element_size(), src.data_ptr(),
                                              src.numel() * src.element_size(), int(level), int(iters), _stream_handle(stream)))
