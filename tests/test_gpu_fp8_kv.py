"""GPU tests of the 8-bit (E4M3) KV cache: the codec bit for bit against the oracle's on every bfloat16 value and every
code, the layer against the oracle's quantised chunked prefill, and the error paths."""
import numpy as np
import pytest
import torch

import synth
from oracle import LayerParams, rel_fro
from oracle.fp8_kv import ChunkedPrefillFp8KV, e4m3_decode, kv_load, kv_store

pytestmark = pytest.mark.gpu
TOL = 1e-2   # relative Frobenius error of a layer output, as for the bfloat16 cache


def R():
    from paper_2509_24381_amd import runner
    return runner


def all_bf16_values():
    return (np.arange(1 << 16, dtype=np.uint32) << 16).view(np.float32)


def same_bits(a, b):
    """float arrays equal element by element, NaN matching NaN, -0 distinct from +0."""
    a = np.asarray(a, dtype=np.float32)
    b = np.asarray(b, dtype=np.float32)
    both_nan = np.isnan(a) & np.isnan(b)
    return bool(np.all(both_nan | (a.view(np.uint32) == b.view(np.uint32))))


@pytest.mark.parametrize("shape_name", ["tiny", "small128"])
@pytest.mark.parametrize("k_scale,v_scale", [(1.0, 1.0), (0.25, 3.0), (float(np.float32(1.0 / 3.0)), 0.0078125)])
def test_store_and_load_agree_with_the_oracle_on_every_bf16_value(shape_name, k_scale, v_scale):
    """Import every bfloat16 bit pattern (NaNs, infinities, denormals, both zeros) as keys and, in another order, as
    values; the stored bytes must be the oracle's codes and the values read back the oracle's, bit for bit."""
    r = R()
    shape = synth.TINY if shape_name == "tiny" else synth.LayerShape("small128", 256, 4, 2, 128, 512)
    stack = r.LayerStack(shape, [synth.layer_weights(shape, 3)], max_tokens=256, max_requests=1, max_pos=1024)
    n = (1 << 16) // (shape.n_kv_heads * shape.head_dim)
    vals = all_bf16_values()
    k = vals.reshape(n, shape.n_kv_heads, shape.head_dim)
    v = vals[np.random.default_rng(1).permutation(1 << 16)].reshape(k.shape)
    kv = stack.new_cache_fp8(n, k_scale, v_scale)
    assert kv.is_fp8 and kv.capacity == n
    to_dev = lambda a: torch.from_numpy(a.copy()).to(device="cuda", dtype=torch.bfloat16)
    kv.import_(0, to_dev(k), to_dev(v))
    ck, cv = (t.cpu().numpy() for t in kv.export_codes(0))
    np.testing.assert_array_equal(ck, kv_store(k, k_scale))
    np.testing.assert_array_equal(cv, kv_store(v, v_scale))
    kb, vb = (r.to_numpy_f32(t) for t in kv.export(0))
    assert same_bits(kb, kv_load(ck, k_scale)) and same_bits(vb, kv_load(cv, v_scale))
    # every code, both operands: the bytes travel unchanged and decode as the format says
    codes = np.arange(256, dtype=np.uint8)
    ck = np.resize(codes, k.shape)
    cv = np.resize(codes[::-1], k.shape)
    kv.import_codes(0, torch.from_numpy(ck).cuda(), torch.from_numpy(cv).cuda())
    back_k, back_v = (t.cpu().numpy() for t in kv.export_codes(0))
    np.testing.assert_array_equal(back_k, ck)
    np.testing.assert_array_equal(back_v, cv)
    kb, vb = (r.to_numpy_f32(t) for t in kv.export(0))
    assert same_bits(kb, kv_load(ck, k_scale)) and same_bits(vb, kv_load(cv, v_scale))
    if k_scale == 1.0:
        assert same_bits(kb, e4m3_decode(ck))


@pytest.mark.parametrize("shape_name,bias", [("tiny", True), ("small128", False)])
def test_layer_on_an_8bit_cache_matches_the_quantised_oracle(shape_name, bias):
    """One request, ragged chunks (a one-row chunk, chunks that end inside a 64-token block, several tiles of keys)."""
    r = R()
    shape = synth.TINY if shape_name == "tiny" else synth.LayerShape("small128", 256, 4, 2, 128, 512)
    w = synth.layer_weights(shape, 41, qkv_bias=bias, gains="uniform")
    cuts = [70, 1, 129, 250, 64, 3]
    n = sum(cuts)
    stack = r.LayerStack(shape, [w], max_tokens=256, max_requests=1, max_pos=1024, qkv_bias=bias, fp8_visible_tokens=n + 64)
    x = synth.prompt_rows([("text", 40), ("image", 300), ("text", n - 340)], shape.hidden, 42)
    k_scale, v_scale = 0.5, 0.125
    kv8 = stack.new_cache_fp8(n, k_scale, v_scale)
    kv16 = stack.new_cache(n)
    st = ChunkedPrefillFp8KV(LayerParams.from_arrays(shape, w), k_scale, v_scale)
    a = 0
    worst = 0.0
    for t in cuts:
        xd = r.to_device_bf16(x[a:a + t])
        y8 = r.to_numpy_f32(stack.prefill_batch(0, [kv8], [t], xd))
        stack.prefill_batch(0, [kv16], [t], xd)
        want = st.prefill_chunk(x[a:a + t])
        worst = max(worst, rel_fro(y8, want))
        a += t
        assert kv8.length(0) == a
    print(f"{shape_name}: worst chunk error {worst:.2e}")
    assert worst <= TOL
    ck, cv = (t.cpu().numpy() for t in kv8.export_codes(0))
    # the same decision in the same precision: the codes are the oracle's encoding of the bfloat16 K~ and V the
    # library itself produced for these rows (what its bfloat16 cache holds) - bit for bit
    k16, v16 = (r.to_numpy_f32(t) for t in kv16.export(0))
    np.testing.assert_array_equal(ck, kv_store(k16, k_scale))
    np.testing.assert_array_equal(cv, kv_store(v16, v_scale))
    # against the oracle's own K~ and V (fp64 from an fp64 RMSNorm, never rounded to bfloat16) a code may land on another
    # value where the two sides' inputs straddle a rounding boundary: rarely, and never further than one step of the
    # format at that magnitude (at most 1/8 of the value) plus the two sides' input difference (bfloat16 rounding of the
    # normalised rows: a few 2^-9 of the typical element)
    for got, want, scale in ((ck, st.codes_k, k_scale), (cv, st.codes_v, v_scale)):
        a_got, a_want = kv_load(got, scale), kv_load(want, scale)
        gap = np.abs(a_got - a_want)
        allowed = np.maximum(np.abs(a_got), np.abs(a_want)) / 8 + np.sqrt(np.mean(a_want ** 2)) * 2.0 ** -6
        print(f"codes differing from the fp64 side's: {np.mean(got != want):.3%}, largest gap / allowed {np.max(gap / allowed):.3f}")
        assert np.mean(got != want) < 0.08 and np.all(gap <= allowed)
    # what attention read: the exported values are the oracle's reading of the library's codes
    k8, v8 = (r.to_numpy_f32(t) for t in kv8.export(0))
    assert same_bits(k8, kv_load(ck, k_scale)) and same_bits(v8, kv_load(cv, v_scale))


def test_chunking_does_not_change_the_stored_codes():
    r = R()
    shape = synth.LayerShape("small128", 256, 4, 2, 128, 512)
    w = synth.layer_weights(shape, 43)
    n = 333
    stack = r.LayerStack(shape, [w], max_tokens=512, max_requests=1, max_pos=1024, fp8_visible_tokens=n + 64)
    x = r.to_device_bf16(synth.prompt_rows([("image", 200), ("text", n - 200)], shape.hidden, 44))
    results = []
    for cuts in ([n], [64, 64, 64, 64, 77], [5, 200, 128]):
        kv = stack.new_cache_fp8(n)
        a = 0
        for t in cuts:
            stack.prefill_batch(0, [kv], [t], x[a:a + t])
            a += t
        results.append([t.cpu().numpy() for t in kv.export_codes(0)])
    for ck, cv in results[1:]:
        np.testing.assert_array_equal(ck, results[0][0])
        np.testing.assert_array_equal(cv, results[0][1])


def test_micro_batches_through_two_layers_on_8bit_caches():
    """Three requests advance in interleaved rounds through a two-layer stack in one rs_prefill_model_batch call per
    round; each request is checked against its own oracle chain (layer outputs rounded to bfloat16 between layers, as
    the library hands them on)."""
    r = R()
    shape = synth.LayerShape("small128", 256, 4, 2, 128, 512)
    ws = [synth.layer_weights(shape, 51 + l, gains="uniform") for l in range(2)]
    lens_total = (300, 517, 130)
    stack = r.LayerStack(shape, ws, max_tokens=512, max_requests=3, max_pos=1024, fp8_visible_tokens=sum(lens_total) + 3 * 64)
    prompts = [synth.prompt_rows([("image", n // 2), ("text", n - n // 2)], shape.hidden, 60 + i) for i, n in enumerate(lens_total)]
    rounds = [[70, 0, 64], [1, 200, 0], [129, 63, 66], [100, 254, 0]]
    assert [sum(c) for c in zip(*rounds)] == list(lens_total)
    kvs = [stack.new_cache_fp8(n, 0.5, 0.25) for n in lens_total]
    params = [LayerParams.from_arrays(shape, w) for w in ws]
    chains = [[ChunkedPrefillFp8KV(p, 0.5, 0.25) for p in params] for _ in prompts]
    done = [0, 0, 0]
    worst = 0.0
    for lens in rounds:
        x = np.concatenate([p[d:d + n] for p, d, n in zip(prompts, done, lens)], axis=0)
        xd = r.to_device_bf16(x)
        y = torch.empty_like(xd)
        stack.ctx.prefill_model_batch(stack.layers, kvs, lens, xd, y, stack.ws)
        got = r.to_numpy_f32(y)
        off = 0
        for i, n in enumerate(lens):
            h = prompts[i][done[i]:done[i] + n]
            for st in chains[i]:
                h = synth.bf16_round(st.prefill_chunk(h).astype(np.float32)) if n else h
            if n:
                worst = max(worst, rel_fro(got[off:off + n], h))
            off += n
            done[i] += n
    print(f"worst request-round error {worst:.2e}")
    assert worst <= TOL
    assert [kv.length(1) for kv in kvs] == list(lens_total)


def test_short_chunk_on_a_long_8bit_cache():
    """4500 cached tokens (imported through the store formula) and a 200-row chunk: the expansion covers 74 blocks and
    the key range is walked in parts."""
    r = R()
    shape = synth.LayerShape("small128", 256, 4, 2, 128, 512)
    w = synth.layer_weights(shape, 71)
    prior, t = 4500, 200
    stack = r.LayerStack(shape, [w], max_tokens=256, max_requests=1, max_pos=8192, fp8_visible_tokens=prior + t + 64)
    rng = np.random.default_rng(72)
    k0 = synth.bf16_round(rng.normal(0, 1.5, (prior, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    v0 = synth.bf16_round(rng.normal(0, 1.0, (prior, shape.n_kv_heads, shape.head_dim)).astype(np.float32))
    kv = stack.new_cache_fp8(prior + t, 1.0, 0.5)
    kv.import_(0, r.to_device_bf16(k0), r.to_device_bf16(v0))
    st = ChunkedPrefillFp8KV(LayerParams.from_arrays(shape, w), 1.0, 0.5)
    st.codes_k, st.codes_v = kv_store(k0, 1.0), kv_store(v0, 0.5)
    st.k, st.v = kv_load(st.codes_k, 1.0), kv_load(st.codes_v, 0.5)
    x = synth.prompt_rows([("text", t)], shape.hidden, 73)
    y = r.to_numpy_f32(stack.prefill_batch(0, [kv], [t], r.to_device_bf16(x)))
    want = st.prefill_chunk(x)
    e = rel_fro(y, want)
    print(f"error {e:.2e}")
    assert e <= TOL
    ck, _ = (c.cpu().numpy() for c in kv.export_codes(0))
    np.testing.assert_array_equal(ck[:prior], st.codes_k[:prior])


def test_error_paths_of_8bit_caches():
    r = R()
    from paper_2509_24381_amd.binding import RsError
    shape = synth.TINY
    w = synth.layer_weights(shape, 81)
    stack = r.LayerStack(shape, [w], max_tokens=128, max_requests=2, max_pos=1024, fp8_visible_tokens=1024)
    ctx = stack.ctx
    x = r.to_device_bf16(synth.prompt_rows([("text", 100)], shape.hidden, 82))
    y = torch.empty_like(x)
    per_token = 4 * shape.n_kv_heads * shape.head_dim      # bf16 K and V of one visible token

    def call(kvs, lens, ws_bytes):
        n = sum(lens)
        ctx.prefill_batch(stack.layers[0], 0, kvs, lens, x[:n], y[:n], stack.ws[:ws_bytes])

    kv8 = stack.new_cache_fp8(1024)
    kv16 = stack.new_cache(256)
    base = ctx.workspace_bytes(100, 1)
    # the expansion of 100 visible tokens is two blocks; one byte less than that is refused and nothing has changed
    with pytest.raises(RsError) as e:
        call([kv8], [100], base)
    assert e.value.status_name == "RS_EWORKSPACE" and kv8.length(0) == 0
    with pytest.raises(RsError) as e:
        call([kv8], [100], base + 128 * per_token - 1)
    assert e.value.status_name == "RS_EWORKSPACE" and kv8.length(0) == 0
    call([kv8], [100], base + 128 * per_token)
    assert kv8.length(0) == 100
    # the need grows with the cache: 200 visible tokens are four blocks
    with pytest.raises(RsError) as e:
        call([kv8], [100], base + 128 * per_token)
    assert e.value.status_name == "RS_EWORKSPACE" and kv8.length(0) == 100
    call([kv8], [100], base + 256 * per_token)
    call([kv8], [0], ctx.workspace_bytes(1, 1))            # an empty chunk expands nothing
    assert kv8.length(0) == 200
    kv8.truncate(0, 20)                                    # ... and shrinks with it
    call([kv8], [100], base + 128 * per_token)
    assert kv8.length(0) == 120
    with pytest.raises(RsError) as e:                      # one kind of cache per call
        call([kv8, kv16], [50, 50], stack.ws.numel())
    assert e.value.status_name == "RS_EINVAL" and kv8.length(0) == 120 and kv16.length(0) == 0
    call([kv16], [50], stack.ws.numel())
    with pytest.raises(RsError) as e:                      # codes exist in 8-bit caches only
        kv16.export_codes(0)
    assert e.value.status_name == "RS_ESTATE"
    torch.cuda.synchronize()


def test_paged_8bit_caches_match_contiguous_ones_bit_for_bit():
    """Three requests of a two-layer stack advance in interleaved rounds on one pool of 8-bit pages, so their pages end up
    scattered; every round's output and every final cache (codes and values) must equal what contiguous 8-bit caches
    give.  Then pages go back to the pool as documented."""
    r = R()
    shape = synth.LayerShape("small128", 256, 4, 2, 128, 512)
    ws = [synth.layer_weights(shape, 91 + l, gains="uniform") for l in range(2)]
    lens_total = (300, 517, 130)
    stack = r.LayerStack(shape, ws, max_tokens=512, max_requests=3, max_pos=1024, fp8_visible_tokens=sum(lens_total) + 3 * 64)
    prompts = [synth.prompt_rows([("image", n // 2), ("text", n - n // 2)], shape.hidden, 95 + i) for i, n in enumerate(lens_total)]
    rounds = [[70, 0, 64], [1, 200, 0], [129, 63, 66], [100, 254, 0]]
    pages_for = lambda t: (t + 63) // 64

    def run(paged):
        pool = stack.new_pool(2 * sum(pages_for(n) for n in lens_total), fp8=True) if paged else None
        kvs = [pool.new_cache(2, 0.5, 0.25) if paged else stack.new_cache_fp8(n, 0.5, 0.25) for n in lens_total]
        assert all(kv.is_fp8 for kv in kvs)
        done = [0, 0, 0]
        outs = []
        for lens in rounds:
            x = r.to_device_bf16(np.concatenate([p[d:d + n] for p, d, n in zip(prompts, done, lens)], axis=0))
            y = torch.empty_like(x)
            stack.ctx.prefill_model_batch(stack.layers, kvs, lens, x, y, stack.ws)
            outs.append(r.to_numpy_f32(y))
            done = [d + n for d, n in zip(done, lens)]
            if paged:
                assert pool.free_pages == pool.pages - 2 * sum(pages_for(d) for d in done)
        codes = [[tuple(t.cpu().numpy() for t in kv.export_codes(l)) for l in range(2)] for kv in kvs]
        values = [[tuple(r.to_numpy_f32(t) for t in kv.export(l)) for l in range(2)] for kv in kvs]
        return outs, codes, values, pool, kvs

    outs_c, codes_c, values_c, _, _ = run(False)
    outs_p, codes_p, values_p, pool, kvs = run(True)
    for a, b in zip(outs_c, outs_p):
        np.testing.assert_array_equal(a, b)
    for ca, cb, va, vb in zip(codes_c, codes_p, values_c, values_p):
        for l in range(2):
            for j in range(2):
                np.testing.assert_array_equal(ca[l][j], cb[l][j])
                assert same_bits(va[l][j], vb[l][j])
    assert pool.page_bytes == 2 * shape.n_kv_heads * 64 * shape.head_dim
    free0 = pool.free_pages
    kvs[1].truncate(0, 130)
    assert pool.free_pages == free0 + pages_for(517) - pages_for(130)
    kvs[1].reset()
    assert pool.free_pages == free0 + 2 * pages_for(517)


def test_paged_8bit_export_import_across_argument_windows_and_pool_limits():
    """16500 tokens need two windows of page numbers in the export / import kernels.  Codes imported into a paged cache come
    back unchanged; values imported through the store formula give the oracle's codes; a chunk on top of them matches a
    contiguous 8-bit cache; the pool refuses what it cannot hold before anything runs."""
    r = R()
    from paper_2509_24381_amd.binding import RsError
    shape = synth.TINY
    w = synth.layer_weights(shape, 101)
    n, t = 16500, 60
    stack = r.LayerStack(shape, [w], max_tokens=64, max_requests=1, max_pos=n + 64, fp8_visible_tokens=n + t + 64)
    rng = np.random.default_rng(102)
    pool = stack.new_pool((n + t + 63) // 64 + 1, fp8=True)
    kv = pool.new_cache(1, 0.25, 0.5)
    ck = rng.integers(0, 0x7F, (n, shape.n_kv_heads, shape.head_dim), dtype=np.uint8)
    cv = rng.integers(0x80, 0xFF, (n, shape.n_kv_heads, shape.head_dim), dtype=np.uint8)
    kv.import_codes(0, torch.from_numpy(ck).cuda(), torch.from_numpy(cv).cuda())
    assert kv.length(0) == n and pool.free_pages == pool.pages - (n + 63) // 64
    bk, bv = (c.cpu().numpy() for c in kv.export_codes(0))
    np.testing.assert_array_equal(bk, ck)
    np.testing.assert_array_equal(bv, cv)
    k = synth.bf16_round(rng.normal(0, 1, ck.shape).astype(np.float32))
    v = synth.bf16_round(rng.normal(0, 1, ck.shape).astype(np.float32))
    kv.import_(0, r.to_device_bf16(k), r.to_device_bf16(v))
    bk, bv = (c.cpu().numpy() for c in kv.export_codes(0))
    np.testing.assert_array_equal(bk, kv_store(k, 0.25))
    np.testing.assert_array_equal(bv, kv_store(v, 0.5))
    flat = stack.new_cache_fp8(n + t, 0.25, 0.5)
    flat.import_codes(0, torch.from_numpy(bk).cuda(), torch.from_numpy(bv).cuda())
    x = r.to_device_bf16(synth.prompt_rows([("text", t)], shape.hidden, 103))
    y_paged = r.to_numpy_f32(stack.prefill_batch(0, [kv], [t], x))
    y_flat = r.to_numpy_f32(stack.prefill_batch(0, [flat], [t], x))
    np.testing.assert_array_equal(y_paged, y_flat)
    assert pool.free_pages == pool.pages - (n + t + 63) // 64
    # the pool has one page left: a second cache may take 64 tokens, not 65 (asked for in two calls of a 64-row budget)
    other = pool.new_cache(1)
    assert pool.free_pages == 1
    stack.prefill_batch(0, [other], [64], torch.cat([x, x[:4]], dim=0))
    with pytest.raises(RsError) as e:
        stack.prefill_batch(0, [other], [1], x[:1])
    assert e.value.status_name == "RS_ECAPACITY" and other.length(0) == 64 and pool.free_pages == 0
    torch.cuda.synchronize()
