"""Hazard check of the fused bf16 kernel's LDS ring.  The release kernel keeps streaming loads in flight across
steps, waits for them with hand-counted vmcnt values and publishes a tile with a single barrier.  A second build
of the same source (FLAT_SYNC_EVERY_PHASE) awaits every load in full and fences every phase with barriers.  If
the release build's synchronisation were too weak anywhere, the two would differ; they must agree bit for bit."""
import ctypes
import os

import numpy as np
import pytest

import paper_2107_06419_amd as fa
from paper_2107_06419_amd import synth
from helpers import to_device

pytestmark = pytest.mark.gpu

SYNC_LIB = os.path.join(os.path.dirname(fa.library_path()), "libflat_attn_sync.so")


def _sync_lib():
    if not os.path.exists(SYNC_LIB):
        pytest.fail(f"{SYNC_LIB} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    import torch  # noqa: F401  (same HIP runtime as the tensors)
    lib = ctypes.CDLL(SYNC_LIB)
    vp, i, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.flat_attn_fwd.restype = i
    lib.flat_attn_fwd.argtypes = [vp, vp, vp, vp, i, i, i, i, f, i, vp]
    lib.flat_attn_fwd_cross.restype = i
    lib.flat_attn_fwd_cross.argtypes = [vp, vp, vp, vp, i, i, i, i, i, f, i, vp, vp]
    return lib


def _both(w, q, k, v):
    import torch
    lib = _sync_lib()
    dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
    rel = torch.full_like(dq, float("nan"))
    chk = torch.full_like(dq, float("nan"))
    fa.flat_attn_fwd(dq, dk, dv, rel, w.scale, w.mask)
    st = torch.cuda.current_stream().cuda_stream
    rc = lib.flat_attn_fwd(dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), chk.data_ptr(), w.B, w.H, w.N, w.d, w.scale, w.mask, st)
    assert rc == 0
    torch.cuda.synchronize()
    return rel, chk


@pytest.mark.parametrize("name", ["cfg2_long_16k", "cfg3_wide_causal_8k"])
def test_release_and_fully_synchronised_builds_agree_at_full_size(name):
    import torch
    w = synth.WORKLOADS[name]
    q, k, v = synth.make_qkv(w)
    print(f"case sync build {name}", flush=True)
    rel, chk = _both(w, q, k, v)
    assert torch.isfinite(rel.float()).all()
    assert torch.equal(rel.view(torch.int16), chk.view(torch.int16))


@pytest.mark.parametrize("d", [32, 64, 96, 128, 256])
@pytest.mark.parametrize("mask", [0, 1])
def test_release_and_fully_synchronised_builds_agree_on_ragged_shapes(d, mask):
    import torch
    for B, H, N in ((1, 2, 33), (2, 3, 1777), (1, 1, 4100)):
        w = synth.custom(f"sync_{d}_{mask}_{N}", B, H, N, d, "bf16", mask, seed=4242 + d + mask + N)
        q, k, v = synth.make_qkv(w)
        print(f"case sync build {w}", flush=True)
        rel, chk = _both(w, q, k, v)
        assert torch.isfinite(rel.float()).all()
        assert torch.equal(rel.view(torch.int16), chk.view(torch.int16))


@pytest.mark.parametrize("H,Nk", [(4, 9000), (300, 3000)])
def test_release_and_fully_synchronised_builds_agree_on_cached_keys(H, Nk):
    """Few queries over many keys with per-batch key counts: short row blocks, long rings.  With 4 heads the launch takes
    the 128-row shape, with 300 heads the 256-row shape of large launches."""
    import torch
    lib = _sync_lib()
    B, Nq, d = 2, 300, 64
    assert fa.flat_attn_tile_shape_default(B, H, Nq, d, 1) == (7 if H == 4 else 0)
    q = synth.tensor_f32((B, H, Nq, d), 77, 0)
    k = synth.tensor_f32((B, H, Nk, d), 77, 1)
    v = synth.tensor_f32((B, H, Nk, d), 77, 2)
    dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
    lens = torch.tensor([Nk, Nk // 2 + 1], dtype=torch.int32, device="cuda")
    rel, chk = torch.full_like(dq, float("nan")), torch.full_like(dq, float("nan"))
    for mask in (0, 1):
        fa.flat_attn_fwd_cross(dq, dk, dv, rel, 0.125, mask, lens)
        rc = lib.flat_attn_fwd_cross(dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), chk.data_ptr(), B, H, Nq, Nk, d, 0.125, mask,
                                     lens.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.isfinite(rel.float()).all()
        assert torch.equal(rel.view(torch.int16), chk.view(torch.int16))


@pytest.mark.parametrize("d", [32, 64, 96, 128, 256])
def test_release_and_fully_synchronised_builds_agree_for_every_tile_shape(d):
    """Every shape of the tile table (other ring depths, wavefront counts and keys per tile than the default) keeps its
    own wait counts and barrier placement, so each is compared with its fully synchronised build."""
    import torch
    lib = _sync_lib()
    vp, i, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.flat_attn_fwd_tile.restype = i
    lib.flat_attn_fwd_tile.argtypes = [vp, vp, vp, vp, i, i, i, i, f, i, i, vp]
    for index in range(fa.flat_attn_tile_shape_count(d)):
        for N, mask in ((1777, 0), (2100, 1)):
            w = synth.custom(f"sync_tile_{d}_{index}_{N}", 1, 3, N, d, "bf16", mask, seed=977 + d + index + N)
            q, k, v = synth.make_qkv(w)
            dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
            rel, chk = torch.full_like(dq, float("nan")), torch.full_like(dq, float("nan"))
            print(f"case sync build tile shape {index} {w}", flush=True)
            fa.flat_attn_fwd_tile(dq, dk, dv, rel, w.scale, w.mask, index)
            rc = lib.flat_attn_fwd_tile(dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), chk.data_ptr(), w.B, w.H, w.N, w.d, w.scale,
                                        w.mask, index, torch.cuda.current_stream().cuda_stream)
            assert rc == 0
            torch.cuda.synchronize()
            assert torch.isfinite(rel.float()).all()
            assert torch.equal(rel.view(torch.int16), chk.view(torch.int16))
