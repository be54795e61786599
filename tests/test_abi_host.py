"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad calls on the host.

No kernel runs here.  On a machine without a GPU rs_ctx_create returns a host-only context, which is enough for every
check that the library makes before launching anything.
"""
import ctypes as C
import os
import re

import pytest

from paper_2509_24381_amd import binding
from paper_2509_24381_amd.binding import Context, LayerConfig, RsError

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        from paper_2509_24381_amd.build import build
        build(verbose=False)
    return binding.load_library()


@pytest.mark.parametrize("header_name, symbols", [("rserve_prefill.h", binding.EXPORTED_SYMBOLS),
                                                  ("rserve_sched.h", binding.SCHED_SYMBOLS)])
def test_header_symbols_are_exported(lib, header_name, symbols):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rs_[a-z_0-9]+)\s*\(", header))
    assert declared == set(symbols)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.rs_version() == 1


def tiny_cfg(**kw):
    base = dict(hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, mlp_inter=1024, max_tokens_per_call=128,
                max_requests=4, max_pos=512)
    base.update(kw)
    return LayerConfig(**base)


@pytest.mark.parametrize("bad", [
    dict(hidden=200), dict(head_dim=96), dict(n_kv_heads=3), dict(mlp_inter=1000), dict(max_tokens_per_call=0),
    dict(hidden=0), dict(rope_theta=-1.0), dict(max_pos=0), dict(hidden=288), dict(mlp_inter=1056),
])
def test_ctx_create_rejects_unsupported_shapes(lib, bad):
    with pytest.raises(RsError) as e:
        Context(tiny_cfg(**bad))
    assert e.value.status_name == "RS_EINVAL"


class FakeDeviceMemory:
    """An aligned integer that stands in for a device pointer; the library must never dereference it on the host."""

    def __init__(self, addr=0x7F0000000000):
        self.addr = addr

    def data_ptr(self):
        return self.addr

    def numel(self):
        return 1 << 40


def make_kv(lib, ctx, n_layers=2, capacity=100, addr=0x7E0000000000):
    h = C.c_void_p()
    nbytes = lib.rs_kv_bytes(ctx.handle, n_layers, capacity)
    st = lib.rs_kv_alloc(ctx.handle, n_layers, capacity, addr, nbytes, C.byref(h))
    assert st == 0, lib.rs_last_error()
    return binding.KVCache(ctx, h.value, None)


def fake_weights(bias=False):
    w = binding._Weights(0x1000, 0x2000, 0x3000 if bias else None, 0x4000, 0x5000, 0x6000, 0x7000)
    return binding.PackedWeights(None, w)


def test_sizes_and_kv_bookkeeping(lib):
    ctx = Context(tiny_cfg())
    # K and V^T planes: capacity rounded up to 64 tokens, Hkv*d*2 bytes per token each, per layer
    assert ctx.kv_bytes(2, 100) == 2 * 2 * 128 * 128 * 2
    assert ctx.kv_bytes(0, 100) == 0
    assert ctx.workspace_bytes(128, 4) >= 128 * (256 + 512 + 256 + 1024) * 2
    assert ctx.workspace_bytes(128, 4) >= ctx.workspace_bytes(64, 2)
    assert ctx.weights_packed_bytes() >= 2 * (512 * 256 + 256 * 256 + 3 * 256 * 1024)
    kv = make_kv(lib, ctx)
    assert kv.capacity == 128 and kv.length(0) == 0 and kv.length(1) == 0
    assert kv.length(2) == -1 and kv.length(-1) == -1
    with pytest.raises(RsError):
        kv.truncate(0, 1)            # longer than the current length
    with pytest.raises(RsError):
        kv.truncate(5, 0)
    kv.truncate(0, 0)
    kv.reset()
    # allocation argument checks
    h = C.c_void_p()
    assert lib.rs_kv_alloc(ctx.handle, 1, 100, 0x7E0000000010, 1 << 30, C.byref(h)) == -1   # misaligned
    assert lib.rs_kv_alloc(ctx.handle, 1, 100, None, 1 << 30, C.byref(h)) == -1
    assert lib.rs_kv_alloc(ctx.handle, 1, 100, 0x7E0000000000, 16, C.byref(h)) == -3          # slab too small
    assert lib.rs_kv_alloc(ctx.handle, 0, 100, 0x7E0000000000, 1 << 30, C.byref(h)) == -1
    assert b"" != lib.rs_last_error()


def test_profile_hook_argument_checks(lib):
    ctx = Context(tiny_cfg())
    assert lib.rs_profile_sample_every(ctx.handle, 0) == -1
    assert lib.rs_profile_sample_every(ctx.handle, -3) == -1
    assert lib.rs_profile_sample_every(None, 2) == -1
    assert lib.rs_profile_sample_every(ctx.handle, 3) == 0
    assert lib.rs_profile_enable(ctx.handle, 99, 4) == -1        # no such step
    assert lib.rs_profile_enable(ctx.handle, 0, 0) == -1         # nothing to measure
    assert lib.rs_profile_enable(ctx.handle, -1, 0) == 0         # switching the hook off needs no device
    ms, n = ctx.profile_read()
    assert (ms, n) == (0.0, 0)


def test_prefill_argument_checks_happen_before_any_launch(lib):
    ctx = Context(tiny_cfg())
    other = Context(tiny_cfg())
    kv = make_kv(lib, ctx)
    kv2 = make_kv(lib, ctx, addr=0x7D0000000000)
    foreign = make_kv(lib, other, addr=0x7C0000000000)
    w = fake_weights()
    mem = FakeDeviceMemory()

    class X:
        def __init__(self, t, addr=0x7B0000000000):
            self.shape = (t, 256)
            self.addr = addr
        def data_ptr(self):
            return self.addr

    def status_of(fn):
        with pytest.raises(RsError) as e:
            fn()
        return e.value.status_name

    # too many rows for one call; chunk larger than the cache; bad layer; foreign cache
    assert status_of(lambda: ctx.prefill_chunk(w, 0, kv, X(129), X(129), mem)) == "RS_EINVAL"
    small = make_kv(lib, ctx, capacity=64, addr=0x7A0000000000)
    assert status_of(lambda: ctx.prefill_chunk(w, 0, small, X(100), X(100), mem)) == "RS_ECAPACITY"
    assert status_of(lambda: ctx.prefill_chunk(w, 2, kv, X(8), X(8), mem)) == "RS_EINVAL"
    assert status_of(lambda: ctx.prefill_chunk(w, 0, foreign, X(8), X(8), mem)) == "RS_ESTATE"
    # misaligned x, null workspace, short workspace
    assert status_of(lambda: ctx.prefill_chunk(w, 0, kv, X(8, 0x7B0000000002), X(8), mem)) == "RS_EINVAL"

    class Short(FakeDeviceMemory):
        def numel(self):
            return 1024
    assert status_of(lambda: ctx.prefill_chunk(w, 0, kv, X(8), X(8), Short())) == "RS_EWORKSPACE"
    # bias requested but missing
    ctx_b = Context(tiny_cfg(qkv_bias=True))
    kv_b = make_kv(lib, ctx_b, addr=0x790000000000)
    assert status_of(lambda: ctx_b.prefill_chunk(w, 0, kv_b, X(8), X(8), mem)) == "RS_EINVAL"
    # batch: duplicate request, negative length, too many requests, budget overflow
    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv, kv], [4, 4], X(8), X(8), mem)) == "RS_EINVAL"
    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv, kv2], [4, -1], X(3), X(3), mem)) == "RS_EINVAL"
    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv] * 5, [1] * 5, X(5), X(5), mem)) == "RS_EINVAL"
    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv, kv2], [100, 100], X(200), X(200), mem)) == "RS_EINVAL"
    # nothing above may have advanced any length
    assert kv.length(0) == 0 and kv2.length(0) == 0 and small.length(0) == 0
    # zero rows is a legal no-op that needs no buffers at all (a request with no schedulable tokens, Algorithm 2)
    ctx.prefill_batch(w, 0, [kv, kv2], [0, 0], X(0, 0), X(0, 0), FakeDeviceMemory(0))
    ctx.prefill_batch(w, 0, [], [], X(0, 0), X(0, 0), FakeDeviceMemory(0))
    assert kv.length(0) == 0


def test_valid_call_without_a_gpu_fails_loudly(lib):
    """On a host without a GPU a call that passes every check must return RS_EHIP, never pretend to have run."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("this check is for GPU-less hosts")
    ctx = Context(tiny_cfg())
    kv = make_kv(lib, ctx)

    class X:
        shape = (8, 256)
        def data_ptr(self):
            return 0x7B0000000000
    with pytest.raises(RsError) as e:
        ctx.prefill_chunk(fake_weights(), 0, kv, X(), X(), FakeDeviceMemory())
    assert e.value.status_name == "RS_EHIP"
    assert kv.length(0) == 0
