"""GPU parity where one tensor is larger than 4 GiB: head offsets beyond 2^31 elements and 2^32 bytes.

The tensors are built on the device from one seeded 64-head block: batch b holds the block with the query rows rolled
by b and the value rows rolled by 3 b + 1, so that every batch gives a different result and a head fetched from the
wrong place cannot pass; the oracle gets the same rolls of the host copy for the sampled heads."""
import numpy as np
import pytest

import oracle
import paper_2107_06419_amd as fa
from paper_2107_06419_amd import synth
from helpers import check_close, sample_rows, to_device, to_host_f64

pytestmark = pytest.mark.gpu


def build(base_q, base_k, base_v, B, dtype):
    import torch
    dq, dk, dv = (to_device(x, dtype) for x in (base_q, base_k, base_v))   # [1, H, N, d]
    Q = torch.empty((B,) + tuple(dq.shape[1:]), dtype=dq.dtype, device="cuda")
    K, V = torch.empty_like(Q), torch.empty_like(Q)
    for b in range(B):
        Q[b] = torch.roll(dq[0], shifts=b, dims=1)
        K[b] = dk[0]
        V[b] = torch.roll(dv[0], shifts=3 * b + 1, dims=1)
    return Q, K, V


def host_head(base_q, base_k, base_v, b, h):
    q = np.roll(base_q[0, h], b, axis=0)[None, None]
    v = np.roll(base_v[0, h], 3 * b + 1, axis=0)[None, None]
    return q.astype(np.float64), base_k[0, h][None, None].astype(np.float64), v.astype(np.float64)


def rounded(shape, seed, tid):
    x = synth.tensor_f32(shape, seed, tid, "normal", 1.0)
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x)).reshape(shape)


@pytest.mark.parametrize("mask", [0, 1])
def test_fused_bf16_tensor_beyond_four_gib(mask):
    import torch
    B, H, N, d = 65, 64, 4096, 128                       # 4160 heads of 1 MiB: 4.06 GiB per tensor
    assert B * H * N * d > 2 ** 31 and B * H * N * d * 2 > 2 ** 32
    base = [rounded((1, H, N, d), 4160, t) for t in range(3)]
    Q, K, V = build(*base, B, "bf16")
    O = torch.full_like(Q, float("nan"))
    scale = float(np.float32(d ** -0.5))
    print(f"case beyond 4 GiB: bf16 B={B} H={H} N={N} d={d} mask={mask}", flush=True)
    fa.flat_attn_fwd(Q, K, V, O, scale, mask)
    torch.cuda.synchronize()
    rows = sample_rows(N, 6, seed=5)
    drows = torch.from_numpy(rows).cuda()
    # heads on both sides of the 2^31-byte, 2^32-byte (= 2^31-element) marks, and the two ends
    for b, h in [(0, 0), (31, 63), (32, 0), (63, 63), (64, 0), (64, 63)]:
        q, k, v = host_head(*base, b, h)
        ref = oracle.attention(q, k, v, scale, mask, rows=rows)
        check_close(to_host_f64(O[b:b + 1, h:h + 1][:, :, drows, :]), ref, "bf16", f"head ({b},{h})")
    assert bool(torch.isfinite(O.view(-1)[-(N * d):].float()).all())


def test_fused_f32_tensor_beyond_four_gib():
    import torch
    B, H, N, d = 520, 64, 512, 64                        # 33280 heads of 128 KiB: 4.06 GiB per tensor
    assert B * H * N * d * 4 > 2 ** 32
    base = [synth.tensor_f32((1, H, N, d), 33280, t, "normal", 1.0) for t in range(3)]
    Q, K, V = build(*base, B, "f32")
    O = torch.full_like(Q, float("nan"))
    print(f"case beyond 4 GiB: f32 B={B} H={H} N={N} d={d}", flush=True)
    fa.flat_attn_fwd_f32(Q, K, V, O, 0.125, 1)
    torch.cuda.synchronize()
    for b, h in [(0, 0), (255, 63), (256, 0), (511, 63), (512, 0), (519, 63)]:
        q, k, v = host_head(*base, b, h)
        ref = oracle.attention(q, k, v, 0.125, 1)
        check_close(to_host_f64(O[b:b + 1, h:h + 1]), ref, "f32", f"head ({b},{h})")


@pytest.mark.parametrize("mask", [0, 1])
def test_cross_and_split_keys_with_a_key_side_beyond_four_gib(mask):
    """Three query rows per head over 65536 keys, 520 heads: K and V are 4.06 GiB each, Q and O tiny."""
    import torch
    B, H, Nq, Nk, d = 65, 8, 3, 65536, 64
    assert B * H * Nk * d * 2 > 2 ** 32
    base_q = rounded((1, H, Nq, d), 520, 0)
    base_k, base_v = rounded((1, H, Nk, d), 520, 1), rounded((1, H, Nk, d), 520, 2)
    dq, dk, dv = (to_device(x, "bf16") for x in (base_q, base_k, base_v))
    Q = torch.stack([torch.roll(dq[0], shifts=b, dims=1) for b in range(B)])
    K = dk.expand(B, H, Nk, d).contiguous()
    V = torch.empty_like(K)
    for b in range(B):
        V[b] = torch.roll(dv[0], shifts=3 * b + 1, dims=1)
    print(f"case beyond 4 GiB: cross / split keys B={B} H={H} Nq={Nq} Nk={Nk} d={d} mask={mask}", flush=True)
    outs = {}
    outs["cross"] = torch.full_like(Q, float("nan"))
    fa.flat_attn_fwd_cross(Q, K, V, outs["cross"], 0.125, mask)
    for n_splits in (0, 5):
        ws = torch.full((fa.flat_attn_fwd_splitkv_workspace_bytes(B, H, Nq, Nk, d, n_splits) // 4,), float("nan"),
                        dtype=torch.float32, device="cuda")
        outs[f"split{n_splits}"] = torch.full_like(Q, float("nan"))
        fa.flat_attn_fwd_splitkv(Q, K, V, outs[f"split{n_splits}"], 0.125, mask, None, n_splits, ws)
    torch.cuda.synchronize()
    for b, h in [(0, 0), (31, 7), (32, 0), (63, 7), (64, 0), (64, 7)]:
        q = np.roll(base_q[0, h], b, axis=0)[None, None].astype(np.float64)
        v = np.roll(base_v[0, h], 3 * b + 1, axis=0)[None, None].astype(np.float64)
        ref = oracle.attention_cross(q, base_k[0, h][None, None].astype(np.float64), v, 0.125, mask)
        for name, out in outs.items():
            check_close(to_host_f64(out[b:b + 1, h:h + 1]), ref, "bf16", f"{name} head ({b},{h})")
