"""GPU parity of the split-keys entry point (few query rows over many keys) against the CPU oracle."""
import numpy as np
import pytest

import oracle
import paper_2107_06419_amd as fa
from paper_2107_06419_amd import synth
from helpers import check_close, to_device, to_host_f64

pytestmark = pytest.mark.gpu


def rounded(shape, seed, tid, mult=1.0):
    x = synth.tensor_f32(shape, seed, tid, "normal", mult)
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x)).reshape(shape)


def run_split(q, k, v, scale, mask, lens, n_splits, poison=True):
    import torch
    B, H, Nq, d = q.shape
    Nk = k.shape[2]
    dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
    out = torch.full_like(dq, float("nan"))
    nbytes = fa.flat_attn_fwd_splitkv_workspace_bytes(B, H, Nq, Nk, d, n_splits)
    assert nbytes > 0
    ws = torch.full((nbytes // 4,), float("nan") if poison else 0.0, dtype=torch.float32, device="cuda")
    kv = None if lens is None else torch.tensor(lens, dtype=torch.int32, device="cuda")
    fa.flat_attn_fwd_splitkv(dq, dk, dv, out, scale, mask, kv, n_splits, ws)
    torch.cuda.synchronize()
    return out


SPLIT_CASES = [  # (B, H, Nq, Nk, kv_lens, n_splits)
    (1, 2, 1, 777, None, 0), (1, 1, 17, 64, None, 4), (2, 2, 100, 3000, [3000, 1500], 5), (1, 3, 300, 5000, None, 0),
    (1, 2, 1000, 1000, None, 3), (1, 2, 640, 1700, None, 7), (2, 1, 257, 4100, [1, 4100], 16), (1, 1, 33, 9000, None, 1),
]


@pytest.mark.parametrize("B,H,Nq,Nk,lens,n_splits", SPLIT_CASES)
@pytest.mark.parametrize("d", [32, 64, 96, 128, 256])
@pytest.mark.parametrize("mask", [0, 1])
def test_splitkv_matches_oracle(B, H, Nq, Nk, lens, n_splits, d, mask):
    seed = 31000 + Nq + Nk + d + mask
    q, k, v = rounded((B, H, Nq, d), seed, 0), rounded((B, H, Nk, d), seed, 1), rounded((B, H, Nk, d), seed, 2)
    scale = float(np.float32(d ** -0.5))
    used = fa.flat_attn_fwd_splitkv_splits(B, H, Nq, Nk, d, n_splits)
    print(f"case splitkv B={B} H={H} Nq={Nq} Nk={Nk} d={d} mask={mask} lens={lens} n_splits={n_splits} -> {used}", flush=True)
    assert 1 <= used <= -(-Nk // (32 if d == 256 else 64))
    out = run_split(q, k, v, scale, mask, lens, n_splits)
    ref = oracle.attention_cross(q, k, v, scale, mask, kv_lens=None if lens is None else np.array(lens))
    check_close(to_host_f64(out), ref, "bf16", "splitkv")


def test_splitkv_peaky_rows_merge_across_very_different_maxima():
    """Keys whose logits grow along the sequence: the splits end with reference maxima hundreds of log2 units apart,
    so the merge has to weight them correctly (and drop the early ones) without overflow."""
    B, H, Nq, Nk, d = 1, 2, 70, 6000, 64
    q = np.abs(rounded((B, H, Nq, d), 5, 0))
    k = np.abs(rounded((B, H, Nk, d), 5, 1))
    ramp = np.linspace(0.1, 6.0, Nk, dtype=np.float32)[None, None, :, None]
    k = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(k * ramp)).reshape(k.shape)
    v = rounded((B, H, Nk, d), 5, 2)
    for mask in (0, 1):
        out = run_split(q, k, v, 0.125, mask, None, 11)
        check_close(to_host_f64(out), oracle.attention_cross(q, k, v, 0.125, mask), "bf16", "splitkv ramp")


@pytest.mark.parametrize("Nq", [1, 64, 256])
def test_splitkv_segment_over_long_cache_full_size(Nq):
    """The launch shape the benchmark times: 16 heads, a segment of Nq new positions over 65536 cached keys, causal."""
    import torch
    B, H, Nk, d = 1, 16, 65536, 64
    q, k, v = rounded((B, H, Nq, d), 77 + Nq, 0), rounded((B, H, Nk, d), 77, 1), rounded((B, H, Nk, d), 77, 2)
    out = run_split(q, k, v, 0.125, 1, None, 0)
    ref = oracle.attention_cross(q, k, v, 0.125, 1)
    check_close(to_host_f64(out), ref, "bf16", f"splitkv long cache Nq={Nq}")
    again = run_split(q, k, v, 0.125, 1, None, 0, poison=False)
    assert torch.equal(out.view(torch.int16), again.view(torch.int16))     # bitwise reproducible, whatever the workspace held
    dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
    one = torch.empty_like(dq)
    fa.flat_attn_fwd_cross(dq, dk, dv, one, 0.125, 1)
    torch.cuda.synchronize()
    check_close(to_host_f64(one), ref, "bf16", "unsplit")
    assert (out.float() - one.float()).abs().max().item() <= 2e-3


def test_splitkv_status_codes_on_device_buffers():
    import torch
    q = torch.zeros(1, 2, 8, 64, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, 2, 900, 64, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros_like(q)
    small = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(fa.FlatAttnError) as e:
        fa.flat_attn_fwd_splitkv(q, k, k, o, 1.0, 0, None, 4, small)
    assert e.value.status == -5
    ws = torch.zeros(fa.flat_attn_fwd_splitkv_workspace_bytes(1, 2, 8, 900, 64, 4) // 4, dtype=torch.float32, device="cuda")
    with pytest.raises(fa.FlatAttnError) as e:
        fa.flat_attn_fwd_splitkv(q, k, k, o, float("nan"), 0, None, 4, ws)
    assert e.value.status == -3
    fa.flat_attn_fwd_splitkv(q, k, k, o, 1.0, 0, None, 4, ws)
    torch.cuda.synchronize()
    assert (o.float() == 0).all()
