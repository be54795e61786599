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
    # a workspace sized for the largest call serves every smaller one: monotone in both arguments
    sizes = [ctx.workspace_bytes(t, 1) for t in range(1, 129)]
    assert all(b >= a for a, b in zip(sizes, sizes[1:]))
    big = Context(tiny_cfg(max_tokens_per_call=1024))
    sizes = [big.workspace_bytes(t, 2) for t in (1, 30, 63, 64, 65, 100, 127, 128, 129, 200, 255, 256, 257, 300, 512, 1000, 1024)]
    assert all(b >= a for a, b in zip(sizes, sizes[1:]))
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


def make_pool(lib, ctx, n_pages, addr=0x700000000000):
    h = C.c_void_p()
    st = lib.rs_kv_pool_create(ctx.handle, addr, n_pages * lib.rs_kv_page_bytes(ctx.handle), C.byref(h))
    assert st == 0, lib.rs_last_error()
    return h


def make_paged_kv(lib, ctx, pool, n_layers=2):
    h = C.c_void_p()
    assert lib.rs_kv_alloc_paged(ctx.handle, pool, n_layers, C.byref(h)) == 0, lib.rs_last_error()
    return binding.KVCache(ctx, h.value, None)


def test_page_pool_bookkeeping_on_the_host(lib):
    """A page = 64 tokens of one layer, K and V of all KV heads.  Pool and paged caches are host bookkeeping until a
    kernel runs, so every rule about pages can be checked without a GPU."""
    ctx = Context(tiny_cfg())
    page = lib.rs_kv_page_bytes(ctx.handle)
    assert page == 2 * 2 * 64 * 64 * 2          # {K, V} x 2 KV heads x 64 tokens x d = 64 x bf16
    h = C.c_void_p()
    assert lib.rs_kv_pool_create(ctx.handle, 0x700000000010, 10 * page, C.byref(h)) == -1   # misaligned
    assert lib.rs_kv_pool_create(ctx.handle, None, 10 * page, C.byref(h)) == -1
    assert lib.rs_kv_pool_create(ctx.handle, 0x700000000000, page - 1, C.byref(h)) == -3    # not even one page
    pool = make_pool(lib, ctx, 5)
    assert lib.rs_kv_pool_pages(pool) == 5 and lib.rs_kv_pool_free_pages(pool) == 5
    assert lib.rs_kv_pool_pages(None) == -1 and lib.rs_kv_pool_free_pages(None) == -1
    assert lib.rs_kv_alloc_paged(ctx.handle, None, 2, C.byref(h)) == -1
    assert lib.rs_kv_alloc_paged(ctx.handle, pool, 0, C.byref(h)) == -1
    stranger = Context(tiny_cfg())
    assert lib.rs_kv_alloc_paged(stranger.handle, pool, 2, C.byref(h)) == -4                 # another context's pool
    kv = make_paged_kv(lib, ctx, pool)
    assert kv.capacity == 0 and kv.length(0) == 0 and lib.rs_kv_pool_free_pages(pool) == 5   # pages come with tokens
    assert lib.rs_kv_pool_destroy(pool) == -4                                                # a cache is alive
    w, mem = fake_weights(), FakeDeviceMemory()

    class X:
        def __init__(self, t):
            self.shape = (t, 256)
        def data_ptr(self):
            return 0x7B0000000000

    def status_of(fn):
        with pytest.raises(RsError) as e:
            fn()
        return e.value.status_name

    # 5 free pages: 128 rows of one layer need 2 pages -> passes every host check (and then misses the GPU here);
    # a second cache asking for 4 more pages in the same call does not fit; nothing is taken by a failing call
    kv2 = make_paged_kv(lib, ctx, pool)
    st = status_of(lambda: ctx.prefill_batch(w, 0, [kv, kv2], [64, 64], X(128), X(128), mem))
    assert st in ("RS_EHIP",)   # enough pages: the call got as far as needing a device
    small = Context(tiny_cfg(max_tokens_per_call=512, max_requests=4))
    pool_s = make_pool(lib, small, 5, addr=0x6F0000000000)
    a, b = make_paged_kv(lib, small, pool_s), make_paged_kv(lib, small, pool_s)
    big = FakeDeviceMemory()
    assert status_of(lambda: small.prefill_batch(w, 0, [a, b], [129, 200], X(329), X(329), big)) == "RS_ECAPACITY"   # 3 + 4 pages
    assert lib.rs_kv_pool_free_pages(pool_s) == 5 and a.length(0) == 0 and a.capacity == 0
    # all layers in one call: 2 layers x 3 pages = 6 > 5, although either layer alone would fit
    assert status_of(lambda: small.prefill_model_batch([w, w], [a], [129], X(129), X(129), big)) == "RS_ECAPACITY"
    assert lib.rs_kv_pool_free_pages(pool_s) == 5
    # the position limit still holds for a cache without a fixed capacity (max_pos = 512 here)
    roomy = make_pool(lib, small, 64, addr=0x6E0000000000)
    c = make_paged_kv(lib, small, roomy)
    assert status_of(lambda: small.prefill_batch(w, 0, [c], [512], X(512), X(512), big)) == "RS_EHIP"       # fits: needs the GPU
    assert lib.rs_kv_import(c.handle, 0, 0x7B0000000000, 0x7B0000100000, 513, None) == -2                   # beyond max_pos
    lib.rs_kv_free(c.handle)
    c.handle = None
    assert lib.rs_kv_pool_destroy(roomy) == 0
    # import: page need is checked before anything else is touched
    assert lib.rs_kv_import(a.handle, 0, 0x7B0000000000, 0x7B0000100000, 64 * 6, None) == -2   # RS_ECAPACITY: 6 pages
    assert lib.rs_kv_import(a.handle, 0, None, None, 0, None) == 0
    assert lib.rs_kv_pool_free_pages(pool_s) == 5
    # freeing the caches lets the pools go
    for c in (kv, kv2, a, b):
        lib.rs_kv_free(c.handle)
        c.handle = None
    assert lib.rs_kv_pool_destroy(pool) == 0 and lib.rs_kv_pool_destroy(pool_s) == 0
    assert lib.rs_kv_pool_destroy(None) == 0


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


def test_static_workspace_entry_point_checks_on_the_host(lib):
    """rs_prefill_chunk_static makes rs_prefill_chunk's checks against the size of the static array: a call beyond it
    is RS_EWORKSPACE (and says which entry point to use instead), one that fits gets as far as needing the GPU."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("this check is for GPU-less hosts")
    assert lib.rs_static_workspace_bytes() == 128 << 20
    cfg7 = LayerConfig(hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, mlp_inter=18944, max_tokens_per_call=2048,
                       max_requests=1, max_pos=4096)
    ctx = Context(cfg7)
    kv = make_kv(lib, ctx, n_layers=1, capacity=4096)

    def X(t):
        class T:
            shape = (t, 3584)
            def data_ptr(self):
                return 0x7B0000000000
        return T()

    def status_of(fn):
        with pytest.raises(RsError) as e:
            fn()
        return e.value
    assert ctx.workspace_bytes(643, 1) <= 128 << 20 < ctx.workspace_bytes(644, 1)
    e = status_of(lambda: ctx.prefill_chunk_static(fake_weights(), 0, kv, X(644), X(644)))
    assert e.status_name == "RS_EWORKSPACE" and "rs_prefill_chunk_static" in str(e)
    assert status_of(lambda: ctx.prefill_chunk_static(fake_weights(), 0, kv, X(643), X(643))).status_name == "RS_EHIP"
    assert status_of(lambda: ctx.prefill_chunk_static(fake_weights(), 3, kv, X(8), X(8))).status_name == "RS_EINVAL"
    assert status_of(lambda: ctx.prefill_chunk_static(fake_weights(), 0, kv, X(4097), X(4097))).status_name == "RS_EINVAL"
    assert lib.rs_prefill_chunk_static(ctx.handle, None, 0, kv.handle, None, 8, None, None) == -1
    assert lib.rs_prefill_chunk_static(ctx.handle, C.byref(fake_weights().struct), 0, None, None, 8, None, None) == -1
    ctx.prefill_chunk_static(fake_weights(), 0, kv, X(0), X(0))   # an empty call is a no-op everywhere
    assert kv.length(0) == 0


def test_8bit_cache_argument_checks_on_the_host(lib):
    """Sizes, scales, the one-kind-per-call rule and the workspace an 8-bit cache's expansion needs: all decided before a
    device is touched."""
    ctx = Context(tiny_cfg())
    assert lib.rs_kv_fp8_bytes(ctx.handle, 2, 100) == ctx.kv_bytes(2, 100) // 2 == 2 * 2 * 128 * 128
    assert lib.rs_kv_fp8_bytes(ctx.handle, 0, 100) == 0 and lib.rs_kv_fp8_bytes(None, 2, 100) == 0
    h = C.c_void_p()
    need = lib.rs_kv_fp8_bytes(ctx.handle, 2, 100)
    for ks, vs in ((0.0, 1.0), (1.0, -1.0), (float("inf"), 1.0), (float("nan"), 1.0), (1.0, 1e-45)):
        assert lib.rs_kv_alloc_fp8(ctx.handle, 2, 100, ks, vs, 0x7D0000000000, need, C.byref(h)) == -1, (ks, vs)
    assert lib.rs_kv_alloc_fp8(ctx.handle, 2, 100, 1.0, 1.0, 0x7D0000000010, need, C.byref(h)) == -1      # misaligned
    assert lib.rs_kv_alloc_fp8(ctx.handle, 2, 100, 1.0, 1.0, 0x7D0000000000, need - 1, C.byref(h)) == -3
    assert lib.rs_kv_alloc_fp8(ctx.handle, 2, 100, 0.5, 2.0, 0x7D0000000000, need, C.byref(h)) == 0, lib.rs_last_error()
    kv8 = binding.KVCache(ctx, h.value, None)
    assert kv8.is_fp8 and kv8.capacity == 128 and kv8.length(1) == 0
    kv16 = make_kv(lib, ctx)
    assert not kv16.is_fp8 and lib.rs_kv_is_fp8(None) == -1
    assert lib.rs_kv_export_codes(kv16.handle, 0, 0x7B0000000000, 0x7B0000100000, None) == -4           # RS_ESTATE
    assert lib.rs_kv_import_codes(kv16.handle, 0, 0x7B0000000000, 0x7B0000100000, 10, None) == -4
    assert lib.rs_kv_import_codes(kv8.handle, 0, 0x7B0000000000, 0x7B0000100000, 129, None) == -2        # beyond capacity
    assert lib.rs_kv_import_codes(kv8.handle, 2, 0x7B0000000000, 0x7B0000100000, 10, None) == -1
    assert lib.rs_kv_import_codes(kv8.handle, 0, None, None, 0, None) == 0
    assert lib.rs_kv_export_codes(kv8.handle, 0, None, None, None) == 0                                 # empty: nothing to do
    # workspace: rs_workspace_bytes plus 4 * Hkv * d bytes per visible token, each request rounded up to 64 tokens
    base = ctx.workspace_bytes(128, 4)
    per_token = 4 * 2 * 64
    assert lib.rs_workspace_bytes_fp8kv(ctx.handle, 128, 4, 0) == base + per_token * 256      # 4 x 63 -> 256 tokens of rounding
    assert lib.rs_workspace_bytes_fp8kv(ctx.handle, 128, 1, 1) == ctx.workspace_bytes(128, 1) + per_token * 64
    assert lib.rs_workspace_bytes_fp8kv(ctx.handle, 128, 1, 65) == ctx.workspace_bytes(128, 1) + per_token * 128
    w = fake_weights()

    class X:
        def __init__(self, t):
            self.shape = (t, 256)
        def data_ptr(self):
            return 0x7B0000000000

    class Mem(FakeDeviceMemory):
        def __init__(self, n):
            super().__init__()
            self.n = n
        def numel(self):
            return self.n

    def status_of(fn):
        with pytest.raises(RsError) as e:
            fn()
        return e.value.status_name

    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv8, kv16], [10, 10], X(20), X(20), Mem(1 << 40))) == "RS_EINVAL"
    ws1 = ctx.workspace_bytes(70, 1)
    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv8], [70], X(70), X(70), Mem(ws1))) == "RS_EWORKSPACE"
    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv8], [70], X(70), X(70), Mem(ws1 + per_token * 128 - 1))) == "RS_EWORKSPACE"
    assert status_of(lambda: ctx.prefill_batch(w, 0, [kv8], [70], X(70), X(70), Mem(ws1 + per_token * 128))) == "RS_EHIP"
    assert kv8.length(0) == 0


def test_8bit_page_pools_on_the_host(lib):
    """An 8-bit pool has half-size pages and serves 8-bit caches only; a bfloat16 pool serves bfloat16 caches only."""
    ctx = Context(tiny_cfg())
    assert lib.rs_kv_page_bytes_fp8(ctx.handle) == lib.rs_kv_page_bytes(ctx.handle) // 2 == 2 * 2 * 64 * 64
    h = C.c_void_p()
    page = lib.rs_kv_page_bytes_fp8(ctx.handle)
    assert lib.rs_kv_pool_create_fp8(ctx.handle, 0x6D0000000000, page - 1, C.byref(h)) == -3
    assert lib.rs_kv_pool_create_fp8(ctx.handle, 0x6D0000000000, 7 * page + 5, C.byref(h)) == 0, lib.rs_last_error()
    pool8 = C.c_void_p(h.value)
    assert lib.rs_kv_pool_pages(pool8) == 7 and lib.rs_kv_pool_is_fp8(pool8) == 1 and lib.rs_kv_pool_is_fp8(None) == -1
    pool16 = make_pool(lib, ctx, 3)
    assert lib.rs_kv_pool_is_fp8(pool16) == 0
    assert lib.rs_kv_alloc_paged(ctx.handle, pool8, 2, C.byref(h)) == -4                       # kinds do not mix
    assert lib.rs_kv_alloc_paged_fp8(ctx.handle, pool16, 2, 1.0, 1.0, C.byref(h)) == -4
    assert lib.rs_kv_alloc_paged_fp8(ctx.handle, pool8, 2, 0.0, 1.0, C.byref(h)) == -1          # scales as for rs_kv_alloc_fp8
    assert lib.rs_kv_alloc_paged_fp8(ctx.handle, pool8, 0, 1.0, 1.0, C.byref(h)) == -1
    assert lib.rs_kv_alloc_paged_fp8(ctx.handle, pool8, 2, 0.5, 2.0, C.byref(h)) == 0, lib.rs_last_error()
    kv = binding.KVCache(ctx, h.value, None)
    assert kv.is_fp8 and kv.capacity == 0 and lib.rs_kv_pool_free_pages(pool8) == 7
    # imports count pages like prefill calls do: 8 pages for 500 tokens, the pool has 7
    assert lib.rs_kv_import_codes(kv.handle, 0, 0x7B0000000000, 0x7B0000100000, 500, None) == -2
    assert lib.rs_kv_import(kv.handle, 0, 0x7B0000000000, 0x7B0000100000, 500, None) == -2
    assert lib.rs_kv_pool_free_pages(pool8) == 7
    assert lib.rs_kv_import_codes(kv.handle, 0, 0x7B0000000000, 0x7B0000100000, 513, None) == -2     # beyond max_pos = 512
    assert lib.rs_kv_pool_destroy(pool8) == -4
    lib.rs_kv_free(kv.handle)
    kv.handle = None
    assert lib.rs_kv_pool_destroy(pool8) == 0 and lib.rs_kv_pool_destroy(pool16) == 0


def test_bench_refuses_more_than_one_gpu():
    """The build is for one GPU: `bench.py --gpus N` with N above 1 exits with status 2 and says why, before it touches a
    device or prints a JSON line."""
    import subprocess
    import sys
    proc = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert proc.returncode == 2
    assert "one GPU" in proc.stderr + proc.stdout
    assert "{" not in proc.stdout
