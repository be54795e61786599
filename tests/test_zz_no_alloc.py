"""rs_prefill_chunk_static (the entry point for callers that cannot allocate: the workspace is a static device array
inside the library) against rs_prefill_chunk with a workspace of the caller's, through the C ABI.

Two calls in a row on the same request, the second with a smaller input: the static array keeps the first call's
intermediates, and nothing in it may leak into the second.  Same kernels, same launch shapes: outputs and caches must be
the same bits; the result is also held to the oracle's bar.  Collected last (the file name sorts after every other test
file): the suite is run with -x, and a failure here must not hide the others.
"""
import numpy as np
import pytest
import torch

import synth
from oracle import LayerParams, layer_forward, rel_fro

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape_name", ["tiny", "small128"])
def test_static_workspace_entry_point_matches_the_caller_workspace_one(shape_name):
    from paper_2509_24381_amd import runner as R
    from paper_2509_24381_amd.binding import RsError
    shape = synth.TINY if shape_name == "tiny" else synth.LayerShape("small128", 512, 8, 2, 128, 768)
    w = synth.layer_weights(shape, 801, qkv_bias=True, gains="uniform")
    t1, t2 = 333, 77                       # the second call is smaller than the first
    x = synth.prompt_rows([("image", 200), ("text", t1 + t2 - 200)], shape.hidden, 802)
    stack = R.LayerStack(shape, [w], max_tokens=512, max_requests=1, max_pos=512, qkv_bias=True)
    assert stack.ctx.static_workspace_bytes() == 128 << 20
    xd = R.to_device_bf16(x)
    kv_a, kv_b = stack.new_cache(t1 + t2), stack.new_cache(t1 + t2)
    y_a, y_b = torch.full_like(xd, float("nan")), torch.full_like(xd, float("nan"))
    for a, b in [(0, t1), (t1, t1 + t2)]:
        stack.ctx.prefill_chunk_static(stack.layers[0], 0, kv_a, xd[a:b], y_a[a:b])
        stack.ctx.prefill_chunk(stack.layers[0], 0, kv_b, xd[a:b], y_b[a:b], stack.ws)
        torch.cuda.synchronize()
        assert kv_a.length(0) == kv_b.length(0) == b
        assert torch.equal(y_a[a:b], y_b[a:b]), f"rows [{a}, {b}) differ between the two entry points"
    (ka, va), (kb, vb) = kv_a.export(0), kv_b.export(0)
    assert torch.equal(ka, kb) and torch.equal(va, vb)
    y_ref, k_ref, v_ref = layer_forward(x, LayerParams.from_arrays(shape, w))
    errs = {"Y": rel_fro(R.to_numpy_f32(y_a), y_ref), "K": rel_fro(R.to_numpy_f32(ka), k_ref), "V": rel_fro(R.to_numpy_f32(va), v_ref)}
    print(f"[parity] static workspace {shape_name}: " + ", ".join(f"{k} {e:.3e}" for k, e in errs.items()), flush=True)
    assert all(e <= 1e-2 for e in errs.values()), errs
    # an empty call is a no-op; a call that does not fit the cache is refused and changes nothing
    stack.ctx.prefill_chunk_static(stack.layers[0], 0, kv_a, xd[:0], y_a[:0])
    room = kv_a.capacity - (t1 + t2)       # (capacities are rounded up to whole 64-token blocks)
    with pytest.raises(RsError) as e:
        stack.ctx.prefill_chunk_static(stack.layers[0], 0, kv_a, xd[:room + 1], y_a[:room + 1])
    assert e.value.status_name == "RS_ECAPACITY" and kv_a.length(0) == t1 + t2


def test_static_workspace_entry_point_refuses_what_it_cannot_hold():
    """A 7B-shaped call of 1024 rows needs more than the 128 MiB the static array holds: RS_EWORKSPACE before anything
    is launched, the cache untouched; 512 rows fit and run."""
    from paper_2509_24381_amd import runner as R
    from paper_2509_24381_amd.binding import RsError
    shape = synth.L7B
    w = synth.layer_weights(shape, 811)
    stack = R.LayerStack(shape, [w], max_tokens=1024, max_requests=1, max_pos=2048)
    assert stack.ctx.workspace_bytes(1024, 1) > stack.ctx.static_workspace_bytes() >= stack.ctx.workspace_bytes(512, 1)
    x = R.to_device_bf16(synth.prompt_rows([("image", 1024)], shape.hidden, 812))
    y = torch.empty_like(x)
    kv = stack.new_cache(2048)
    with pytest.raises(RsError) as e:
        stack.ctx.prefill_chunk_static(stack.layers[0], 0, kv, x, y)
    assert e.value.status_name == "RS_EWORKSPACE" and "static workspace" in str(e.value) and kv.length(0) == 0
    kv_b = stack.new_cache(2048)
    y_b = torch.empty_like(x)
    stack.ctx.prefill_chunk_static(stack.layers[0], 0, kv, x[:512], y[:512])
    stack.ctx.prefill_chunk(stack.layers[0], 0, kv_b, x[:512], y_b[:512], stack.ws)
    torch.cuda.synchronize()
    assert kv.length(0) == 512 and torch.equal(y[:512], y_b[:512])
