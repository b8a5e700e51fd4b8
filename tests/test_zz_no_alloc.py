"""The allocation-free split-keys entry point (flat_attn_fwd_splitkv_static) against the workspace form it is a
variant of: same kernels, so with the same number of splits the two must agree bit for bit.  Two calls in a row share
the library's built-in scratch buffer, the second with a smaller input, so stale partial results of the first call
would show."""
import numpy as np
import pytest

import oracle
import paper_2107_06419_amd as fa
from paper_2107_06419_amd import synth
from helpers import check_close, to_device, to_host_f64

pytestmark = pytest.mark.gpu


def rounded(shape, seed, tid):
    x = synth.tensor_f32(shape, seed, tid, "normal", 1.0)
    return synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x)).reshape(shape)


def both_forms(B, H, Nq, Nk, d, mask, lens, n_splits, seed):
    import torch
    q, k, v = rounded((B, H, Nq, d), seed, 0), rounded((B, H, Nk, d), seed, 1), rounded((B, H, Nk, d), seed, 2)
    dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
    kv = None if lens is None else torch.tensor(lens, dtype=torch.int32, device="cuda")
    scale = float(np.float32(d ** -0.5))
    used = fa.flat_attn_fwd_splitkv_splits(B, H, Nq, Nk, d, n_splits)
    ws = torch.full((fa.flat_attn_fwd_splitkv_workspace_bytes(B, H, Nq, Nk, d, n_splits) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    with_ws = torch.full_like(dq, float("nan"))
    fa.flat_attn_fwd_splitkv(dq, dk, dv, with_ws, scale, mask, kv, n_splits, ws)
    static = torch.full_like(dq, float("nan"))
    print(f"case no-alloc B={B} H={H} Nq={Nq} Nk={Nk} d={d} mask={mask} lens={lens} splits={used}", flush=True)
    fa.flat_attn_fwd_splitkv_static(dq, dk, dv, static, scale, mask, kv, used)
    torch.cuda.synchronize()
    ref = oracle.attention_cross(q, k, v, scale, mask, kv_lens=None if lens is None else np.array(lens))
    return with_ws, static, ref


def test_static_scratch_form_equals_the_workspace_form_on_two_calls_in_a_row():
    import torch
    # first call: large (the partial results fill 38 MiB of the 64 MiB buffer); second call: smaller in every dimension
    for args in ((1, 16, 256, 20000, 64, 1, None, 36, 901), (2, 3, 70, 3000, 128, 0, [3000, 1234], 5, 902), (1, 2, 1, 500, 256, 1, None, 0, 903)):
        with_ws, static, ref = both_forms(*args)
        assert torch.equal(with_ws.view(torch.int16), static.view(torch.int16))
        check_close(to_host_f64(static), ref, "bf16", f"no-alloc {args}")


def test_static_scratch_form_refuses_what_does_not_fit():
    import torch
    q = torch.zeros(1, 16, 256, 64, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, 16, 65536, 64, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros_like(q)
    with pytest.raises(fa.FlatAttnError) as e:
        fa.flat_attn_fwd_splitkv_static(q, k, k, o, 0.125, 1, None, 64)      # 16 * 64 * 256 * 66 * 4 bytes = 66 MiB
    assert e.value.status == -5
    fa.flat_attn_fwd_splitkv_static(q, k, k, o, 0.125, 1, None, 0)           # the library's choice is cut to what fits
    torch.cuda.synchronize()
    assert (o.float() == 0).all()


def test_static_scratch_form_replays_from_a_hip_graph():
    """What the entry point is for: captured into a HIP graph (nothing in it allocates or clears memory) and replayed,
    with eager work between the replays; every replay equals the eager result bit for bit."""
    import torch
    B, H, Nq, Nk, d = 1, 8, 40, 6000, 64
    q, k, v = rounded((B, H, Nq, d), 77, 0), rounded((B, H, Nk, d), 77, 1), rounded((B, H, Nk, d), 77, 2)
    dq, dk, dv = (to_device(x, "bf16") for x in (q, k, v))
    eager = torch.empty_like(dq)
    fa.flat_attn_fwd_splitkv_static(dq, dk, dv, eager, 0.125, 1, None, 0)    # also resolves the buffer's address before the capture
    torch.cuda.synchronize()
    check_close(to_host_f64(eager), oracle.attention_cross(q, k, v, 0.125, 1), "bf16", "no-alloc eager")
    out = torch.zeros_like(dq)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fa.flat_attn_fwd_splitkv_static(dq, dk, dv, out, 0.125, 1, None, 0, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        out.fill_(float("nan"))
        other = torch.empty(B, H, 300, d, dtype=torch.bfloat16, device="cuda")
        fa.flat_attn_fwd_splitkv_static(dk[:, :, :300].contiguous(), dk, dv, other, 0.125, 0, None, 3)   # eager use of the same buffer
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
