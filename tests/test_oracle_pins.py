"""Pins for the fp64 oracle: each piece is checked against something other than itself.

The paper prints no worked numeric example of the layer, so the pins are brute force on tiny
inputs, library routines on special cases, closed forms and invariants the paper states
(section 2.2.1: a chunk depends on earlier chunks only through the KV cache, hence chunked
prefill must equal unchunked prefill for any chunking).
"""
import math
from types import SimpleNamespace

import numpy as np
import pytest
import torch

import oracle
from oracle import (ChunkedPrefill, LayerParams, attention_loops, causal_gqa_attention,
                    layer_forward, layer_forward_rows, prefill_batch, rel_fro, rmsnorm, rope, silu)
from oracle.decoder_layer import _softmax_rows  # noqa: F401  (row-sum pin)


def small_params(rng, hidden=32, hq=4, hkv=2, d=8, inter=48, bias=False, std=0.3, gains=True):
    shape = SimpleNamespace(hidden=hidden, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, mlp_inter=inter,
                            rms_eps=1e-6, rope_theta=1e4)
    w = SimpleNamespace(
        g1=rng.uniform(0.5, 1.5, hidden) if gains else np.ones(hidden),
        g2=rng.uniform(0.5, 1.5, hidden) if gains else np.ones(hidden),
        wq=rng.normal(0, std, (hq * d, hidden)), wk=rng.normal(0, std, (hkv * d, hidden)),
        wv=rng.normal(0, std, (hkv * d, hidden)), wo=rng.normal(0, std, (hidden, hq * d)),
        wg=rng.normal(0, std, (inter, hidden)), wu=rng.normal(0, std, (inter, hidden)),
        wd=rng.normal(0, std, (hidden, inter)),
        bq=rng.normal(0, std, hq * d) if bias else None,
        bk=rng.normal(0, std, hkv * d) if bias else None,
        bv=rng.normal(0, std, hkv * d) if bias else None)
    return LayerParams.from_arrays(shape, w)


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("n,hq,hkv,d", [(1, 2, 1, 4), (7, 4, 2, 6), (19, 6, 2, 8), (33, 3, 3, 4)])
def test_attention_matches_scalar_loops(n, hq, hkv, d):
    rng = np.random.default_rng(n * 100 + hq)
    q = rng.normal(size=(n, hq, d))
    k = rng.normal(size=(n, hkv, d))
    v = rng.normal(size=(n, hkv, d))
    out, probs = causal_gqa_attention(q, k, v, return_probs=True, row_block=5)
    ref_out, ref_probs = attention_loops(q.tolist(), k.tolist(), v.tolist())
    np.testing.assert_allclose(out, np.array(ref_out), rtol=0, atol=1e-12)
    np.testing.assert_allclose(probs, np.array(ref_probs), rtol=0, atol=1e-13)


def test_attention_matches_library_sdpa():
    rng = np.random.default_rng(11)
    n, hq, hkv, d = 48, 8, 2, 16
    q = rng.normal(size=(n, hq, d))
    k = rng.normal(size=(n, hkv, d))
    v = rng.normal(size=(n, hkv, d))
    g = hq // hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).repeat_interleave(g, dim=1).permute(1, 0, 2)[None]
    tv = torch.from_numpy(v).repeat_interleave(g, dim=1).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(causal_gqa_attention(q, k, v), ref, rtol=0, atol=1e-12)


def test_attention_closed_forms():
    rng = np.random.default_rng(5)
    n, hq, hkv, d = 12, 4, 2, 8
    q = rng.normal(size=(n, hq, d))
    v = rng.normal(size=(n, hkv, d))
    # identical keys -> uniform weights over the visible prefix -> running mean of V
    k_same = np.broadcast_to(rng.normal(size=(1, hkv, d)), (n, hkv, d)).copy()
    out = causal_gqa_attention(q, k_same, v)
    running_mean = np.cumsum(v, axis=0) / np.arange(1, n + 1)[:, None, None]
    for h in range(hq):
        np.testing.assert_allclose(out[:, h], running_mean[:, h // 2], atol=1e-13)
    # a single token attends only to itself
    out1 = causal_gqa_attention(q[:1], rng.normal(size=(1, hkv, d)), v[:1])
    for h in range(hq):
        np.testing.assert_allclose(out1[0, h], v[0, h // 2], atol=1e-15)
    # constant V -> constant output
    k = rng.normal(size=(n, hkv, d))
    vc = np.broadcast_to(rng.normal(size=(1, hkv, d)), (n, hkv, d)).copy()
    outc = causal_gqa_attention(q, k, vc)
    for h in range(hq):
        np.testing.assert_allclose(outc[:, h], np.broadcast_to(vc[0, h // 2], (n, d)), atol=1e-13)


def test_attention_is_causal_and_rows_sum_to_one():
    rng = np.random.default_rng(6)
    n, hq, hkv, d = 20, 4, 2, 8
    q, k, v = (rng.normal(size=s) for s in [(n, hq, d), (n, hkv, d), (n, hkv, d)])
    out, probs = causal_gqa_attention(q, k, v, return_probs=True)
    assert np.max(np.abs(probs.sum(-1) - 1.0)) <= 1e-12
    assert np.all(np.triu(probs, k=1) == 0.0)
    assert np.all(probs >= 0.0)
    cut = 9
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[cut + 1:] += 3.0
    k2[cut + 1:] -= 2.0
    v2[cut + 1:] *= -5.0
    out2 = causal_gqa_attention(q2, k2, v2)
    assert np.array_equal(out[: cut + 1], out2[: cut + 1])
    assert not np.allclose(out[cut + 1:], out2[cut + 1:])


def test_gqa_equals_expanded_mha_and_head_mapping():
    rng = np.random.default_rng(7)
    n, hq, hkv, d = 10, 6, 3, 4
    q, k, v = (rng.normal(size=s) for s in [(n, hq, d), (n, hkv, d), (n, hkv, d)])
    g = hq // hkv
    out = causal_gqa_attention(q, k, v)
    out_mha = causal_gqa_attention(q, np.repeat(k, g, axis=1), np.repeat(v, g, axis=1))
    np.testing.assert_allclose(out, out_mha, atol=1e-14)
    # head h must read KV head h//g (consecutive query heads share a KV head), not h % Hkv:
    v_mark = np.zeros_like(v)
    v_mark[:, 1, :] = 1.0
    out_mark = causal_gqa_attention(q, k, v_mark)
    for h in range(hq):
        expect = 1.0 if h // g == 1 else 0.0
        np.testing.assert_allclose(out_mark[:, h], expect, atol=1e-14)


def test_scale_is_inverse_sqrt_head_dim():
    # two keys with scores differing by exactly ln(3)*sqrt(d) -> weights 1/4, 3/4
    d = 16
    q = np.zeros((2, 1, d)); q[:, 0, 0] = 1.0
    k = np.zeros((2, 1, d)); k[1, 0, 0] = math.log(3.0) * math.sqrt(d)
    v = np.zeros((2, 1, d)); v[0, 0, 0] = 1.0; v[1, 0, 1] = 1.0
    out = causal_gqa_attention(q, k, v)
    np.testing.assert_allclose(out[1, 0, :2], [0.25, 0.75], atol=1e-14)
    np.testing.assert_allclose(out[0, 0, :2], [1.0, 0.0], atol=1e-15)


# ------------------------------------------------------------------ RoPE
def test_rope_properties():
    rng = np.random.default_rng(8)
    n, h, d, theta = 9, 3, 16, 1e6
    v = rng.normal(size=(n, h, d))
    pos = np.array([0, 1, 2, 5, 17, 100, 4097, 32767, 31])
    r = rope(v, pos, theta)
    np.testing.assert_array_equal(r[0], v[0])                              # position 0 is the identity
    np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-13)
    # complex form: (v_j + i v_{j+d/2}) * exp(i * pos * theta^(-2j/d))
    j = np.arange(d // 2)
    phase = np.exp(1j * pos[:, None] * theta ** (-2.0 * j / d))[:, None, :]
    z = (v[..., : d // 2] + 1j * v[..., d // 2:]) * phase
    np.testing.assert_allclose(r[..., : d // 2], z.real, atol=1e-10)
    np.testing.assert_allclose(r[..., d // 2:], z.imag, atol=1e-10)
    # printed-by-hand value: d=2, theta arbitrary -> plain 2-D rotation by pos radians
    r2 = rope(np.array([[[1.0, 0.0]]]), np.array([1]), 10.0)
    np.testing.assert_allclose(r2[0, 0], [math.cos(1.0), math.sin(1.0)], atol=1e-15)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(9)
    d, theta = 32, 1e6
    q = rng.normal(size=(1, 1, d))
    k = rng.normal(size=(1, 1, d))
    def score(n, m):
        return float(np.sum(rope(q, np.array([n]), theta) * rope(k, np.array([m]), theta)))
    base = score(40, 25)
    for shift in (1, 77, 1000, 20000):
        assert abs(score(40 + shift, 25 + shift) - base) < 1e-8
    assert abs(score(41, 25) - base) > 1e-3


def test_rope_frequency_of_second_pair():
    # d=4, theta=100: pair j=1 rotates by pos * 100^(-2/4) = pos / 10
    v = np.zeros((1, 1, 4)); v[0, 0, 1] = 1.0
    r = rope(v, np.array([5]), 100.0)
    np.testing.assert_allclose(r[0, 0], [0.0, math.cos(0.5), 0.0, math.sin(0.5)], atol=1e-15)


# ------------------------------------------------------------------ RMSNorm / SiLU / GEMM
def test_rmsnorm_pins():
    rng = np.random.default_rng(10)
    x = rng.normal(size=(5, 64)) * 3.0
    g = rng.uniform(0.5, 1.5, 64)
    out1 = rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(out1 ** 2, axis=-1)), 1.0, rtol=1e-13)
    np.testing.assert_allclose(rmsnorm(7.5 * x, g, 0.0), rmsnorm(x, g, 0.0), rtol=1e-13)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-6).numpy()
    np.testing.assert_allclose(rmsnorm(x, g, 1e-6), ref, rtol=1e-13)
    # eps sits inside the square root: x = 0 row stays 0, and a tiny row is damped by sqrt(eps)
    tiny = np.full((1, 4), 1e-6)
    np.testing.assert_allclose(rmsnorm(tiny, np.ones(4), 1e-6), tiny / math.sqrt(1e-12 + 1e-6), rtol=1e-13)
    # hand value: [3, 4] -> mean square 12.5
    np.testing.assert_allclose(rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0),
                               [[3 / math.sqrt(12.5), 8 / math.sqrt(12.5)]], rtol=1e-15)


def test_silu_matches_library_and_hand_values():
    z = np.linspace(-20, 20, 101)
    np.testing.assert_allclose(silu(z), torch.nn.functional.silu(torch.from_numpy(z)).numpy(), rtol=1e-13, atol=1e-300)
    assert silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(silu(np.array([1.0]))[0], 1.0 / (1.0 + math.exp(-1.0)), rtol=1e-15)


def test_projection_is_x_times_w_transposed():
    rng = np.random.default_rng(12)
    p = small_params(rng, hidden=6, hq=2, hkv=1, d=4, inter=5, bias=True)
    x = rng.normal(size=(3, 6))
    from oracle.decoder_layer import _project_qkv
    q, k, v = _project_qkv(x, p)
    for n in range(3):
        for o in range(8):
            want = sum(x[n, i] * p.wq[o, i] for i in range(6)) + p.bq[o]
            assert abs(q.reshape(3, 8)[n, o] - want) < 1e-13
        for o in range(4):
            want_k = sum(x[n, i] * p.wk[o, i] for i in range(6)) + p.bk[o]
            want_v = sum(x[n, i] * p.wv[o, i] for i in range(6)) + p.bv[o]
            assert abs(k.reshape(3, 4)[n, o] - want_k) < 1e-13
            assert abs(v.reshape(3, 4)[n, o] - want_v) < 1e-13


# ------------------------------------------------------------------ whole layer
def torch_layer(x, p: LayerParams):
    """The layer recomposed from torch library routines (fp64), RoPE via complex multiplication."""
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    X = t(x)
    n = X.shape[0]
    h = F.rms_norm(X, (p.hidden,), t(p.g1), eps=p.rms_eps)
    q = F.linear(h, t(p.wq), None if p.bq is None else t(p.bq)).view(n, p.n_q_heads, p.head_dim)
    k = F.linear(h, t(p.wk), None if p.bk is None else t(p.bk)).view(n, p.n_kv_heads, p.head_dim)
    v = F.linear(h, t(p.wv), None if p.bv is None else t(p.bv)).view(n, p.n_kv_heads, p.head_dim)
    half = p.head_dim // 2
    inv = torch.pow(torch.tensor(p.rope_theta, dtype=torch.float64),
                    -torch.arange(0, half, dtype=torch.float64) * 2.0 / p.head_dim)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * inv[None, :]
    phase = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    def rot(a):
        z = torch.complex(a[..., :half], a[..., half:]) * phase
        return torch.cat([z.real, z.imag], dim=-1)
    q, k = rot(q), rot(k)
    o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None],
                                       is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).reshape(n, -1)
    r = X + F.linear(o, t(p.wo))
    h2 = F.rms_norm(r, (p.hidden,), t(p.g2), eps=p.rms_eps)
    y = r + F.linear(F.silu(F.linear(h2, t(p.wg))) * F.linear(h2, t(p.wu)), t(p.wd))
    return y.numpy(), k.numpy(), v.numpy()


@pytest.mark.parametrize("bias", [False, True])
def test_layer_matches_library_composition(bias):
    rng = np.random.default_rng(13)
    p = small_params(rng, hidden=48, hq=6, hkv=2, d=8, inter=80, bias=bias)
    x = rng.normal(size=(37, 48))
    y, k, v = layer_forward(x, p)
    ry, rk, rv = torch_layer(x, p)
    np.testing.assert_allclose(y, ry, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(k, rk, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(v, rv, rtol=1e-10, atol=1e-11)


def test_layer_residual_special_cases():
    rng = np.random.default_rng(14)
    p = small_params(rng)
    x = rng.normal(size=(11, p.hidden))
    p.wd = np.zeros_like(p.wd)
    y, _, _ = layer_forward(x, p)
    # W_d = 0: the MLP adds nothing, Y is the attention residual; with W_o = 0 as well Y = X
    h = rmsnorm(x, p.g1, p.rms_eps)
    from oracle.decoder_layer import _project_qkv
    q, k, v = _project_qkv(h, p)
    o = causal_gqa_attention(rope(q, np.arange(11), p.rope_theta), rope(k, np.arange(11), p.rope_theta), v)
    np.testing.assert_allclose(y, x + o.reshape(11, -1) @ p.wo.T, atol=1e-13)
    p.wo = np.zeros_like(p.wo)
    y2, _, _ = layer_forward(x, p)
    np.testing.assert_array_equal(y2, x)


def test_layer_fp32_rerun_agrees():
    """Conditioning check: the same layer in float32 torch stays within ~1e-5 of the fp64 oracle."""
    rng = np.random.default_rng(15)
    p = small_params(rng, hidden=64, hq=4, hkv=2, d=16, inter=128, std=0.1)
    x = rng.normal(size=(40, 64))
    y, _, _ = layer_forward(x, p)
    p32 = LayerParams(**{k: (v.astype(np.float32).astype(np.float64) if isinstance(v, np.ndarray) else v)
                         for k, v in p.__dict__.items()})
    y32, _, _ = layer_forward(x.astype(np.float32).astype(np.float64), p32)
    assert rel_fro(y32, y) < 1e-5


def test_rows_form_equals_full_form():
    rng = np.random.default_rng(16)
    p = small_params(rng, bias=True)
    x = rng.normal(size=(29, p.hidden))
    y, k, v = layer_forward(x, p)
    rows = [0, 1, 7, 28, 13]
    yr, kr, vr = layer_forward_rows(x, p, rows)
    np.testing.assert_allclose(yr, y[rows], atol=1e-12)
    np.testing.assert_allclose(kr, k, atol=1e-13)
    np.testing.assert_allclose(vr, v, atol=1e-13)
    # every row, out of order and with a repeat, in slabs of 1, 4 and all at once: the slabs only bound memory
    rows = list(rng.permutation(29)) + [5]
    for row_block in (1, 4, 64):
        yr, _, _ = layer_forward_rows(x, p, rows, row_block=row_block)
        np.testing.assert_allclose(yr, y[rows], atol=1e-12)


# ------------------------------------------------------------------ chunking / batching (section 2.2.1, Algorithm 2)
def random_partition(rng, n):
    cuts = sorted(set(rng.integers(1, n, size=rng.integers(0, 6)).tolist()))
    edges = [0] + cuts + [n]
    return [(a, b) for a, b in zip(edges[:-1], edges[1:])]


@pytest.mark.parametrize("seed", range(6))
def test_chunked_equals_unchunked(seed):
    rng = np.random.default_rng(100 + seed)
    p = small_params(rng, bias=bool(seed % 2))
    n = int(rng.integers(8, 60))
    x = rng.normal(size=(n, p.hidden)) * np.where(rng.random((n, 1)) < 0.5, 1.0, 0.02)  # image-like / text-like rows
    y, k, v = layer_forward(x, p)
    partitions = [random_partition(rng, n), [(0, n)], [(i, i + 1) for i in range(n)]]
    for part in partitions:
        st = ChunkedPrefill(p)
        outs = [st.prefill_chunk(x[a:b]) for a, b in part]
        assert st.length == n
        assert rel_fro(np.concatenate(outs), y) <= 1e-10
        assert rel_fro(st.k, k) <= 1e-10
        assert rel_fro(st.v, v) <= 1e-10
        np.testing.assert_allclose(np.concatenate(outs), y, rtol=0, atol=1e-10)


def test_chunk_with_zero_rows_is_a_noop():
    rng = np.random.default_rng(20)
    p = small_params(rng)
    st = ChunkedPrefill(p)
    st.prefill_chunk(rng.normal(size=(5, p.hidden)))
    k_before = st.k.copy()
    out = st.prefill_chunk(np.zeros((0, p.hidden)))
    assert out.shape == (0, p.hidden) and st.length == 5
    np.testing.assert_array_equal(st.k, k_before)


def test_batch_equals_per_request_loop_and_permutes():
    rng = np.random.default_rng(21)
    p = small_params(rng)
    priors = [0, 9, 3, 17]
    lens = [4, 1, 0, 6]
    reqs = []
    for pr, t in zip(priors, lens):
        reqs.append((rng.normal(size=(pr, p.n_kv_heads, p.head_dim)), rng.normal(size=(pr, p.n_kv_heads, p.head_dim)),
                     rng.normal(size=(t, p.hidden))))
    def run(order):
        states = [ChunkedPrefill(p, reqs[i][0], reqs[i][1]) for i in order]
        y = prefill_batch(states, [reqs[i][2] for i in order])
        return y, states
    y, states = run([0, 1, 2, 3])
    # looping prefill_chunk per request
    off = 0
    for i, (pk, pv, rows) in enumerate(reqs):
        st = ChunkedPrefill(p, pk, pv)
        yi = st.prefill_chunk(rows)
        np.testing.assert_array_equal(y[off: off + lens[i]], yi)
        np.testing.assert_array_equal(states[i].k, st.k)
        assert states[i].length == priors[i] + lens[i]
        off += lens[i]
    # permuting the requests permutes the packed output blocks and nothing else
    order = [3, 0, 2, 1]
    yp, _ = run(order)
    starts = np.concatenate([[0], np.cumsum(lens)])
    offp = 0
    for i in order:
        np.testing.assert_array_equal(yp[offp: offp + lens[i]], y[starts[i]: starts[i] + lens[i]])
        offp += lens[i]
    with pytest.raises(ValueError):
        st = ChunkedPrefill(p)
        prefill_batch([st, st], [reqs[0][2], reqs[0][2]])


def test_prior_cache_continuation_matches_full_prompt():
    """A state seeded with the K~/V of the first P tokens continues exactly like the full prompt."""
    rng = np.random.default_rng(22)
    p = small_params(rng)
    x = rng.normal(size=(23, p.hidden))
    y, k, v = layer_forward(x, p)
    st = ChunkedPrefill(p, k[:15], v[:15])
    out = st.prefill_chunk(x[15:])
    np.testing.assert_allclose(out, y[15:], atol=1e-11)
    np.testing.assert_allclose(st.k, k, atol=1e-12)


def test_chunk_attention_matches_scalar_loops_with_prefix():
    """The chunk-vs-prefix mask (prefix fully visible, chunk causal) against explicit loops."""
    rng = np.random.default_rng(23)
    p = small_params(rng, hidden=16, hq=4, hkv=2, d=4, inter=8)
    p.wo = np.eye(16)          # expose the attention output in r
    p.wd = np.zeros_like(p.wd)
    prior, t = 6, 5
    pk = rng.normal(size=(prior, 2, 4)); pv = rng.normal(size=(prior, 2, 4))
    x = rng.normal(size=(t, 16))
    st = ChunkedPrefill(p, pk, pv)
    y = st.prefill_chunk(x)
    from oracle.decoder_layer import _project_qkv
    h = rmsnorm(x, p.g1, p.rms_eps)
    q, kn, vn = _project_qkv(h, p)
    pos = prior + np.arange(t)
    q = rope(q, pos, p.rope_theta); kn = rope(kn, pos, p.rope_theta)
    o, _ = attention_loops(q.tolist(), np.concatenate([pk, kn]).tolist(), np.concatenate([pv, vn]).tolist(), n_prior=prior)
    np.testing.assert_allclose(y - x, np.array(o).reshape(t, 16), atol=1e-12)


def test_first_token_logits_closed_form_on_one_hot_rows():
    """x = c e_k: mean(x^2) = c^2/H, so rmsnorm(x) = sign(c) sqrt(H) / sqrt(1 + eps H / c^2) g_k e_k and the logits are
    that factor times column k of w_lm; a constant row with unit gain gives the row sums of w_lm (eps -> 0)."""
    import oracle
    rng = np.random.default_rng(77)
    h, vocab, eps = 48, 19, 1e-6
    g = rng.uniform(0.5, 1.5, h)
    w = rng.standard_normal((vocab, h))
    for k, c in ((0, 2.0), (17, -0.3), (47, 1e-2)):
        x = np.zeros((1, h))
        x[0, k] = c
        want = np.sign(c) * np.sqrt(h) / np.sqrt(1.0 + eps * h / c ** 2) * g[k] * w[:, k]
        np.testing.assert_allclose(oracle.first_token_logits(x, g, w, eps)[0], want, rtol=1e-12, atol=1e-12)
    got = oracle.first_token_logits(np.full((2, h), 3.0), np.ones(h), w, 0.0)
    np.testing.assert_allclose(got, np.tile(w.sum(axis=1), (2, 1)), rtol=1e-12)
    # rows are independent, and the result is linear in w_lm
    x = rng.standard_normal((3, h))
    a = oracle.first_token_logits(x, g, w, eps)
    np.testing.assert_allclose(oracle.first_token_logits(x[1:2], g, w, eps), a[1:2], rtol=1e-13)
    np.testing.assert_allclose(oracle.first_token_logits(x, g, 2.0 * w, eps), 2.0 * a, rtol=1e-13)


def test_three_axis_rope_reduces_to_1d_and_turns_each_pair_by_its_axis():
    """(1) equal positions on the three axes, or a single section, give the 1-D rotation (up to rounding order); (2) pair j, written
    out as a scalar complex multiplication, turns by the position of the axis whose section holds j; (3) norms are
    kept; (4) scores depend only on per-axis position differences."""
    import oracle
    rng = np.random.default_rng(88)
    n, heads, d, theta = 9, 3, 32, 1e4
    sections = (4, 8, 4)
    v = rng.standard_normal((n, heads, d))
    pos = rng.integers(0, 50, size=n)
    same = np.stack([pos, pos, pos], axis=1)
    np.testing.assert_allclose(oracle.rope(v, same, theta, sections), oracle.rope(v, pos, theta), rtol=1e-12, atol=1e-13)
    p3 = rng.integers(0, 50, size=(n, 3))
    np.testing.assert_allclose(oracle.rope(v, p3, theta, (16, 0, 0)), oracle.rope(v, p3[:, 0], theta), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.rope(v, p3, theta, (0, 0, 16)), oracle.rope(v, p3[:, 2], theta), rtol=1e-12, atol=1e-13)
    out = oracle.rope(v, p3, theta, sections)
    axis_of = [0] * 4 + [1] * 8 + [2] * 4
    for t in range(n):
        for j in range(d // 2):
            ang = p3[t, axis_of[j]] * theta ** (-2.0 * j / d)
            z = (v[t, 1, j] + 1j * v[t, 1, j + d // 2]) * np.exp(1j * ang)
            assert abs(out[t, 1, j] - z.real) < 1e-12 and abs(out[t, 1, j + d // 2] - z.imag) < 1e-12
    np.testing.assert_allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(v, axis=-1), rtol=1e-13)
    q, k = rng.standard_normal((2, n, 1, d))
    base = np.einsum("nhd,mhd->nm", oracle.rope(q, p3, theta, sections), oracle.rope(k, p3, theta, sections))
    shift = np.array([7, 0, 3])
    moved = np.einsum("nhd,mhd->nm", oracle.rope(q, p3 + shift, theta, sections), oracle.rope(k, p3 + shift, theta, sections))
    np.testing.assert_allclose(moved, base, rtol=1e-10, atol=1e-10)
