"""GPU edge cases of the C ABI: limits, aliasing, poisoned buffers, cache bookkeeping, both kernel variants."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import synth
from oracle import ChunkedPrefill, LayerParams, layer_forward, prefill_batch, rel_fro

pytestmark = pytest.mark.gpu
TOL = 1e-2
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def R():
    from paper_2509_24381_amd import runner
    return runner


def check(name, got, want, tol=TOL):
    err = rel_fro(got, want)
    print(f"[parity] {name}: rel_fro = {err:.3e}", flush=True)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    assert err <= tol, f"{name}: rel_fro {err:.3e} > {tol}"


def test_poisoned_buffers_exact_capacity_and_in_place_output():
    """KV slab and workspace start as NaN bit patterns; the chunk sizes end exactly at capacity; y aliases x.

    Nothing the kernels read may depend on uninitialised memory (the V cache's zero tail is maintained by the append
    kernel), the cache must hold exactly `capacity` tokens, and writing the output over the input must be safe."""
    r = R()
    shape = synth.TINY
    w = synth.layer_weights(shape, 5, gains="uniform")
    n = 192                                   # capacity is a multiple of 64: the cache is filled to its last slot
    x = synth.prompt_rows([("image", 100), ("text", 92)], shape.hidden, 6)
    stack = r.LayerStack(shape, [w], max_tokens=100, max_requests=2, max_pos=n)
    kv = stack.new_cache(n)
    assert kv.capacity == n
    kv.slab.view(torch.int16).fill_(0x7FC1)      # bf16 NaN pattern everywhere
    stack.ws.view(torch.int16).fill_(0x7FC1)
    xd = r.to_device_bf16(x)
    buf = xd.clone()
    for a, b in [(0, 100), (100, 133), (133, 192)]:
        stack.ctx.prefill_chunk(stack.layers[0], 0, kv, buf[a:b], buf[a:b], stack.ws)   # in place
    torch.cuda.synchronize()
    assert kv.length(0) == n
    y_ref, k_ref, v_ref = layer_forward(x, LayerParams.from_arrays(shape, w))
    k, v = kv.export(0)
    check("poisoned Y (in place)", r.to_numpy_f32(buf), y_ref)
    check("poisoned K", r.to_numpy_f32(k), k_ref)
    check("poisoned V", r.to_numpy_f32(v), v_ref)
    # one more row does not fit
    from paper_2509_24381_amd.binding import RsError
    with pytest.raises(RsError) as e:
        stack.ctx.prefill_chunk(stack.layers[0], 0, kv, xd[:1], buf[:1], stack.ws)
    assert e.value.status_name == "RS_ECAPACITY" and kv.length(0) == n


def test_truncate_then_refill_matches_fresh_prefill():
    """Dropping the newest tokens and prefilling them again reproduces the cache and the output bit for bit."""
    r = R()
    shape = synth.TINY
    w = synth.layer_weights(shape, 8)
    x = synth.prompt_rows([("text", 70), ("image", 90)], shape.hidden, 9)
    stack = r.LayerStack(shape, [w], max_tokens=160, max_requests=1, max_pos=256)
    kv = stack.new_cache(200)
    xd = r.to_device_bf16(x)
    y1 = torch.empty_like(xd)
    stack.ctx.prefill_chunk(stack.layers[0], 0, kv, xd[:100], y1[:100], stack.ws)
    stack.ctx.prefill_chunk(stack.layers[0], 0, kv, xd[100:], y1[100:], stack.ws)
    torch.cuda.synchronize()
    k1, v1 = kv.export(0)
    kv.truncate(0, 100)
    assert kv.length(0) == 100
    y2 = torch.empty_like(xd[100:])
    stack.ctx.prefill_chunk(stack.layers[0], 0, kv, xd[100:], y2, stack.ws)
    torch.cuda.synchronize()
    k2, v2 = kv.export(0)
    assert torch.equal(y2, y1[100:]) and torch.equal(k1, k2) and torch.equal(v1, v2)
    kv.reset()
    assert kv.length(0) == 0


def test_single_rows_against_long_prefix_and_full_budget_call():
    """T = 1 calls (the smallest legal chunk) against a growing prefix, then one call that uses the whole token budget."""
    r = R()
    shape = synth.LayerShape("s", 256, 8, 2, 64, 512)
    w = synth.layer_weights(shape, 12, qkv_bias=True, gains="uniform")
    n = 700
    x = synth.prompt_rows([("image", 300), ("text", 400)], shape.hidden, 13)
    stack = r.LayerStack(shape, [w], max_tokens=512, max_requests=1, max_pos=1024, qkv_bias=True)
    kv = stack.new_cache(n)
    xd = r.to_device_bf16(x)
    y = torch.empty_like(xd)
    chunks = [(0, 183)] + [(i, i + 1) for i in range(183, 188)] + [(188, 700)]    # 512 = the whole budget
    for a, b in chunks:
        stack.ctx.prefill_chunk(stack.layers[0], 0, kv, xd[a:b], y[a:b], stack.ws)
    torch.cuda.synchronize()
    y_ref, k_ref, v_ref = layer_forward(x, LayerParams.from_arrays(shape, w))
    k, v = kv.export(0)
    check("T=1 / full budget Y", r.to_numpy_f32(y), y_ref)
    check("T=1 rows only", r.to_numpy_f32(y)[183:188], y_ref[183:188])
    check("T=1 / full budget K", r.to_numpy_f32(k), k_ref)
    check("T=1 / full budget V", r.to_numpy_f32(v), v_ref)


def test_batch_at_request_limit_with_mixed_capacities_is_order_equivariant():
    """R = max_requests, caches of different capacities, permuting the requests permutes the output blocks only."""
    r = R()
    shape = synth.TINY
    w = synth.layer_weights(shape, 21)
    rng = np.random.default_rng(22)
    n_req = 8
    priors = [0, 7, 64, 65, 127, 128, 200, 31]
    lens = [9, 1, 30, 2, 17, 64, 3, 2]
    caps = [64, 64, 128, 128, 192, 192, 256, 64]
    reqs = []
    for p, t in zip(priors, lens):
        pk = synth.bf16_round(rng.standard_normal((p, 2, 64), dtype=np.float32))
        pv = synth.bf16_round(rng.standard_normal((p, 2, 64), dtype=np.float32))
        rows = synth.bf16_round(rng.standard_normal((t, 256), dtype=np.float32))
        reqs.append(synth.BatchRequest(p, pk, pv, rows))
    stack = r.LayerStack(shape, [w], max_tokens=sum(lens), max_requests=n_req, max_pos=256)

    def run(order):
        kvs = []
        for i in order:
            kv = stack.new_cache(caps[i])
            if reqs[i].prior_len:
                kv.import_(0, r.to_device_bf16(reqs[i].prior_k), r.to_device_bf16(reqs[i].prior_v))
            kvs.append(kv)
        x = np.concatenate([reqs[i].rows for i in order])
        y = stack.prefill_batch(0, kvs, [lens[i] for i in order], r.to_device_bf16(x))
        torch.cuda.synchronize()
        return r.to_numpy_f32(y), [tuple(r.to_numpy_f32(t_) for t_ in kv.export(0)) for kv in kvs]

    order = list(range(n_req))
    y, caches = run(order)
    p = LayerParams.from_arrays(shape, w)
    states = [ChunkedPrefill(p, q.prior_k, q.prior_v) for q in reqs]
    y_ref = prefill_batch(states, [q.rows for q in reqs])
    check("limit batch Y", y, y_ref)
    for i, st in enumerate(states):
        check(f"limit batch K req {i}", caches[i][0], st.k)
        check(f"limit batch V req {i}", caches[i][1], st.v)
    perm = [5, 0, 7, 2, 6, 1, 4, 3]
    yp, caches_p = run(perm)
    starts = np.concatenate([[0], np.cumsum(lens)])
    off = 0
    for slot, i in enumerate(perm):
        np.testing.assert_array_equal(yp[off: off + lens[i]], y[starts[i]: starts[i] + lens[i]])
        np.testing.assert_array_equal(caches_p[slot][0], caches[i][0])
        np.testing.assert_array_equal(caches_p[slot][1], caches[i][1])
        off += lens[i]


def test_profile_hook_counts_and_samples_launches():
    """rs_profile_enable brackets a step's launches with events; rs_profile_sample_every thins them out; neither changes
    the result."""
    r = R()
    shape = synth.TINY
    w = synth.layer_weights(shape, 41)
    x = r.to_device_bf16(synth.prompt_rows([("text", 256)], shape.hidden, 42))
    stack = r.LayerStack(shape, [w], max_tokens=64, max_requests=1, max_pos=256)
    chunks = [(0, 64), (64, 128), (128, 192), (192, 256)]

    def run(step, every):
        kv = stack.new_cache(256)
        stack.ctx.profile_enable(step, 16, every=every)
        y = stack.prefill_prompt(x, chunks, kv)
        torch.cuda.synchronize()
        ms, n = stack.ctx.profile_read()
        stack.ctx.profile_enable(None)
        return r.to_numpy_f32(y), ms, n

    y0, ms0, n0 = run(None, 1)
    assert (ms0, n0) == (0.0, 0)
    y1, ms1, n1 = run("gate_up_gemm", 1)
    assert n1 == 4 and ms1 > 0.0
    y2, ms2, n2 = run("attention", 3)       # launches 0 and 3 of the four
    assert n2 == 2 and ms2 > 0.0
    np.testing.assert_array_equal(y1, y0)
    np.testing.assert_array_equal(y2, y0)


def test_many_calls_in_flight_on_changing_streams():
    """The library stages each call's descriptors in a ring of pinned buffers and reuses a buffer only when the call that
    used it has consumed it; that is tracked with an event every few calls and at every change of stream.  A hundred
    short calls with different chunk lengths are issued without waiting, on three streams in an irregular pattern (each
    cache stays on one stream); every output must equal, bit for bit, that of the same calls issued one at a time."""
    r = R()
    shape = synth.TINY
    w = synth.layer_weights(shape, 51)
    stack = r.LayerStack(shape, [w], max_tokens=64, max_requests=1, max_pos=4096)
    workspaces = [stack.ctx.workspace(64, 1) for _ in range(3)]        # one per stream: calls on different streams overlap
    streams = [torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.current_stream()]
    rng = np.random.default_rng(52)
    lens = rng.integers(1, 65, size=100).tolist()
    which = [int(v) for v in rng.choice(3, size=100, p=[0.45, 0.35, 0.2])]
    for i in range(20, 40):
        which[i] = 0                                                  # a long run on one stream: periodic checkpoints only
    xs = [r.to_device_bf16(synth.prompt_rows([("text", n)], shape.hidden, 1000 + i)) for i, n in enumerate(lens)]

    def run(serial):
        kvs = [stack.new_cache(4096) for _ in range(3)]
        ys = [torch.empty_like(x) for x in xs]
        torch.cuda.synchronize()
        for i, (n, sidx) in enumerate(zip(lens, which)):
            with torch.cuda.stream(streams[sidx]):
                stack.ctx.prefill_chunk(stack.layers[0], 0, kvs[sidx], xs[i], ys[i], workspaces[sidx], stream=streams[sidx])
            if serial:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        return [r.to_numpy_f32(y) for y in ys], [kv.length(0) for kv in kvs]

    ys_serial, lens_serial = run(True)
    ys_async, lens_async = run(False)
    assert lens_serial == lens_async == [sum(n for n, s in zip(lens, which) if s == k) for k in range(3)]
    for i, (a, b) in enumerate(zip(ys_serial, ys_async)):
        np.testing.assert_array_equal(a, b, err_msg=f"call {i} (T={lens[i]}, stream {which[i]})")


def test_export_import_round_trip_is_bit_exact():
    r = R()
    shape = synth.LayerShape("s128", 256, 2, 1, 128, 256)
    w = synth.layer_weights(shape, 30)
    stack = r.LayerStack(shape, [w, w], max_tokens=64, max_requests=1, max_pos=512)
    rng = np.random.default_rng(31)
    for n in (1, 63, 64, 65, 300):
        k = synth.bf16_round(rng.standard_normal((n, 1, 128), dtype=np.float32))
        v = synth.bf16_round(rng.standard_normal((n, 1, 128), dtype=np.float32))
        kv = stack.new_cache(320)
        kv.import_(1, r.to_device_bf16(k), r.to_device_bf16(v))
        assert kv.length(1) == n and kv.length(0) == 0
        k2, v2 = kv.export(1)
        np.testing.assert_array_equal(r.to_numpy_f32(k2), k)
        np.testing.assert_array_equal(r.to_numpy_f32(v2), v)


def test_a_capturing_stream_is_refused_and_nothing_changes():
    """Calls stage their descriptors through host memory that later calls reuse, so a recorded call would replay with
    stale ones: on a stream that is capturing a HIP graph the library returns RS_ESTATE before it launches or changes
    anything (a paged cache keeps its pages in the pool), and works as before once the capture is over."""
    r = R()
    from paper_2509_24381_amd.binding import RsError
    shape = synth.TINY
    w = synth.layer_weights(shape, 61)
    stack = r.LayerStack(shape, [w], max_tokens=128, max_requests=1, max_pos=512)
    pool = stack.new_pool(4)
    kv = pool.new_cache(1)
    x = r.to_device_bf16(synth.prompt_rows([("text", 100)], shape.hidden, 62))
    y = torch.empty_like(x)
    stack.prefill_batch(0, [kv], [30], x[:30], y[:30])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    status = None
    with torch.cuda.graph(g):
        try:
            stack.prefill_batch(0, [kv], [70], x[30:], y[30:])
        except RsError as e:
            status = e.status_name
    assert status == "RS_ESTATE" and kv.length(0) == 30 and pool.free_pages == 3
    y2 = stack.prefill_batch(0, [kv], [70], x[30:], y[30:])
    torch.cuda.synchronize()
    fresh = stack.new_cache(100)
    y_ref = torch.empty_like(x)
    stack.prefill_batch(0, [fresh], [30], x[:30], y_ref[:30])
    stack.prefill_batch(0, [fresh], [70], x[30:], y_ref[30:])
    torch.cuda.synchronize()
    assert kv.length(0) == 100 and torch.equal(y, y_ref)


@pytest.mark.parametrize("shape_name", ["small128", "wide_mlp"])
def test_row_counts_around_every_wavefront_and_block_boundary(shape_name):
    """The GEMMs choose their geometry and the work of their wavefronts by the row count of the call: wavefronts whose 64
    rows lie past the end idle, calls of 129 to 256 rows on narrow strips run in blocks of 128 rows with the units of a
    pair split between wavefronts, longer calls in blocks of 256.  One call per row count on a prior cache of 100 tokens,
    each against the oracle, and each bit-identical to the same rows taken from a longer call (a row's result does not
    depend on how many rows the call has)."""
    r = R()
    shape = (synth.LayerShape("small128", 256, 4, 2, 128, 512) if shape_name == "small128"
             else synth.LayerShape("wide_mlp", 512, 8, 2, 64, 4096))
    w = synth.layer_weights(shape, 77, qkv_bias=True, gains="uniform")
    stack = r.LayerStack(shape, [w], max_tokens=512, max_requests=1, max_pos=1024, qkv_bias=True)
    prior, longest = 100, 400
    x = synth.prompt_rows([("text", prior), ("image", longest)], shape.hidden, 78)
    params = LayerParams.from_arrays(shape, w)
    base = ChunkedPrefill(params)
    base.prefill_chunk(x[:prior])
    kv = stack.new_cache(prior + longest)
    stack.prefill_batch(0, [kv], [prior], r.to_device_bf16(x[:prior]))
    xd = r.to_device_bf16(x[prior:])
    y_long = r.to_numpy_f32(stack.prefill_batch(0, [kv], [longest], xd))
    k_long, v_long = (r.to_numpy_f32(t) for t in kv.export(0))
    st = ChunkedPrefill(params, prior_k=base.k, prior_v=base.v)
    want_long = st.prefill_chunk(x[prior:])
    check("400 rows", y_long, want_long)
    for t in (1, 31, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 300):
        kv.truncate(0, prior)
        y = r.to_numpy_f32(stack.prefill_batch(0, [kv], [t], xd[:t]))
        check(f"{t} rows", y, want_long[:t])
        k, v = (r.to_numpy_f32(c) for c in kv.export(0))
        # K~ and V of a row come out of the QKV GEMM alone: the same bits whatever the call's row count
        np.testing.assert_array_equal(k, k_long[:prior + t])
        np.testing.assert_array_equal(v, v_long[:prior + t])


@pytest.mark.parametrize("shape_name", ["tiny", "small128"])
def test_a_request_alone_and_next_to_another_leaves_the_same_bits(shape_name):
    """The same request, alone in its calls and next to a second request of one row, must leave the same bits in its
    cache and in its output rows, chunk after chunk (chunk ends off every block, wavefront and 8-token boundary; qkv bias
    on, so that rows past a call's last would not come out as zeros), and the V^T places behind the last token of a block
    must read as zeros although the slab started as NaN patterns."""
    r = R()
    shape = synth.TINY if shape_name == "tiny" else synth.LayerShape("small128", 512, 8, 2, 128, 768)
    w = synth.layer_weights(shape, 911, qkv_bias=True, gains="uniform")
    cuts = [0, 70, 71, 135, 391, 448, 449, 700]
    x = synth.prompt_rows([("image", 300), ("text", 400)], shape.hidden, 912)
    other = synth.prompt_rows([("text", 8)], shape.hidden, 913)
    stack = r.LayerStack(shape, [w], max_tokens=512, max_requests=2, max_pos=1024, qkv_bias=True)
    xd, od = r.to_device_bf16(x), r.to_device_bf16(other)
    kv_a, kv_b, kv_o = stack.new_cache(704), stack.new_cache(704), stack.new_cache(64)
    for kv in (kv_a, kv_b):
        kv.slab.view(torch.int16).fill_(0x7FC1)
    for i, (a, b) in enumerate(zip(cuts[:-1], cuts[1:])):
        y_a = stack.prefill_batch(0, [kv_a], [b - a], xd[a:b])
        y_b = stack.prefill_batch(0, [kv_b, kv_o], [b - a, 1], torch.cat([xd[a:b], od[i:i + 1]]))
        torch.cuda.synchronize()
        np.testing.assert_array_equal(r.to_numpy_f32(y_a), r.to_numpy_f32(y_b)[:b - a])
        assert torch.equal(kv_a.slab.view(torch.int16), kv_b.slab.view(torch.int16)) or _same_up_to(kv_a, kv_b, b, shape)
        for kv in (kv_a, kv_b):
            k, v = kv.export(0)
            assert k.shape[0] == b
    k_a, v_a = (r.to_numpy_f32(t) for t in kv_a.export(0))
    k_b, v_b = (r.to_numpy_f32(t) for t in kv_b.export(0))
    np.testing.assert_array_equal(k_a, k_b)
    np.testing.assert_array_equal(v_a, v_b)
    y_ref, k_ref, v_ref = layer_forward(x, LayerParams.from_arrays(shape, w))
    check("K of the request alone", k_a, k_ref)
    check("V of the request alone", v_a, v_ref)


def _same_up_to(kv_a, kv_b, n, shape):
    """The two slabs agree wherever the layout defines content: K rows below n, and whole V^T blocks up to the one that
    holds token n - 1 (zero tail included).  (K rows at and beyond n are never read and keep whatever they held.)"""
    cap, hkv, d = kv_a.capacity, shape.n_kv_heads, shape.head_dim
    a = kv_a.slab.view(torch.int16).flatten()[: 2 * hkv * cap * d]
    b = kv_b.slab.view(torch.int16).flatten()[: 2 * hkv * cap * d]
    ka, kb = a[: hkv * cap * d].view(hkv, cap, d), b[: hkv * cap * d].view(hkv, cap, d)
    va, vb = a[hkv * cap * d:].view(hkv, cap // 64, d, 64), b[hkv * cap * d:].view(hkv, cap // 64, d, 64)
    nb = (n + 63) // 64
    tail_zero = bool((va[:, nb - 1, :, (n - 1) % 64 + 1:] == 0).all())
    return bool(torch.equal(ka[:, :n], kb[:, :n]) and torch.equal(va[:, :nb], vb[:, :nb]) and tail_zero)


def test_attention_item_order_does_not_change_a_bit(monkeypatch):
    """Between one and two attention blocks per compute unit the host pairs heavy blocks with light ones by compute unit
    instead of launching them heaviest-first.  Blocks are independent, so the two orders must agree to the bit.  The
    compute-unit count is a context setting read from the environment when the context is created: 7 here, so that the
    12 blocks of a 384-row chunk (6 blocks of 128 stacked rows x 2 KV heads) fall between 7 and 14."""
    r = R()
    shape = synth.TINY
    w = synth.layer_weights(shape, 921, gains="uniform")
    x = r.to_device_bf16(synth.prompt_rows([("image", 500), ("text", 268)], shape.hidden, 922))
    outs = []
    for order in ("plain", None):
        monkeypatch.setenv("RS_NCU", "7")
        if order:
            monkeypatch.setenv("RS_ATTN_ORDER", order)
        else:
            monkeypatch.delenv("RS_ATTN_ORDER", raising=False)
        stack = r.LayerStack(shape, [w], max_tokens=384, max_requests=1, max_pos=1024)
        kv = stack.new_cache(768)
        y = stack.prefill_prompt(x, [(0, 384), (384, 768)], kv)
        torch.cuda.synchronize()
        outs.append(r.to_numpy_f32(y))
    np.testing.assert_array_equal(outs[0], outs[1])
    y_ref, _, _ = layer_forward(r.to_numpy_f32(x), LayerParams.from_arrays(shape, w))
    check("paired order Y", outs[1], y_ref)


@pytest.mark.parametrize("env", [{"RS_SPLITK": "1"}, {"RS_SPLITK": "2"}, {"RS_SPLITK": "3"},
                                 {"RS_NCU": "1"}, {"RS_NCU": "3"}, {"RS_NCU": "7", "RS_SPLITK": "2"},
                                 {"RS_ATTN_SPLIT": "1"}, {"RS_ATTN_SPLIT": "3"}, {"RS_ATTN_ORDER": "plain", "RS_NCU": "7"},
                                 {"RS_NARROW": "0"}, {"RS_NARROW": "1", "RS_NARROW_TM": "8", "RS_NCU": "40"}, {"RS_PAIRS": "0"}])
def test_alternative_kernel_paths_meet_the_same_bar(env):
    """Other split-K factors of the residual GEMMs, and other numbers of strips (RS_NCU stands in for the device's
    compute-unit count: small values give wide strips, i.e. every tile width from 2 to 8 units on these small shapes,
    where the default gives one unit per strip), and a fixed number of parts per attention block (RS_ATTN_SPLIT: 1 never splits a key
    range, 3 cuts every block with at least 48 key tiles in three and those with at least 32 in two), and the GEMM geometry
    for launches whose strips hold at most two units (RS_NARROW 0: never the narrow one; RS_NARROW_TM 8: also for calls of
    up to 8 token blocks, which with RS_NCU 40 makes strips of one and two units on these shapes; RS_PAIRS 0: never two
    wavefronts per pair of units), and the plain order of the attention work items (RS_ATTN_ORDER; the default order, which
    depends on the compute-unit count, also runs under every RS_NCU value above) are selectable by
    environment variable; each must pass the
    workload-1 parity test on its own (run in a child process because the choice is read once per process)."""
    child_env = dict(os.environ, **env)
    proc = subprocess.run([sys.executable, "-m", "pytest", "-q", "-x", os.path.join(ROOT, "tests", "test_gpu_parity.py"),
                           os.path.join(ROOT, "tests", "test_gpu_paged_kv.py"), os.path.join(ROOT, "tests", "test_gpu_fp8_kv.py"),
                           "-k", "workload1 or small_ragged or two_layers or odd_head or bit_for_bit or splits_the_key or growing "
                                 "or long_8bit or quantised_oracle"],
                          cwd=ROOT, env=child_env, capture_output=True, text=True, timeout=600)
    assert proc.returncode == 0, proc.stdout[-2000:] + proc.stderr[-2000:]
