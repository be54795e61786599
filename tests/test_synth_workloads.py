"""Host-side checks of the seeded input generators (no layer arithmetic lives there)."""
import numpy as np
import torch

import synth
from synth import L7B, L72B, TINY, bf16_bits, bf16_round, bits_to_f32, workload


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4096).astype(np.float32) * s for s in (1e-3, 1.0, 300.0)])
    # exact ties: mantissa pattern ...1000_0000_0000_0000 must round to even
    ties = (np.arange(256, dtype=np.uint32) << 16 | 0x3F800000 | 0x8000).view(np.float32)
    x = np.concatenate([x, ties, -ties])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bf16_bits(x), want)
    np.testing.assert_array_equal(bf16_round(x), torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    np.testing.assert_array_equal(bf16_bits(bits_to_f32(want)), want)


def test_shapes_and_flop_constants():
    # per-token linear FLOPs and weight bytes of the two production shapes
    assert L7B.linear_flops_per_token() == 466_092_032
    assert L72B.linear_flops_per_token() == 1_755_316_224
    assert TINY.linear_flops_per_token() == 1_966_080
    assert L7B.group == 7 and L72B.group == 8 and TINY.group == 2
    assert L7B.qkv_dim == 4608 and L72B.qkv_dim == 10240 and TINY.qkv_dim == 512
    assert L7B.attn_flops(1, 0) == 14336 and L72B.attn_flops(1, 0) == 32768 and TINY.attn_flops(1, 0) == 1024


def test_workload_layouts():
    w1, w2, w3, w5 = workload(1), workload(2), workload(3), workload(5)
    assert (w1.n_tokens, w1.budget, len(w1.chunks())) == (512, 128, 4)
    assert (w2.n_tokens, w2.budget, len(w2.chunks())) == (2048, 512, 4)
    assert (w3.n_tokens, w3.budget, len(w3.chunks()), w3.n_layers) == (8192, 2048, 4, 4)
    assert sum(n for k, n in w3.segments if k == "image") == 6 * 1024
    assert w3.segments[-1] == ("text", 768)
    assert (w5.n_tokens, w5.budget, len(w5.chunks())) == (32768, 4096, 8)
    assert w5.chunks()[-1] == (28672, 32768)
    x = w1.prompt()
    assert x.shape == (512, 256)
    assert 0.9 < x[:256].std() < 1.1 and 0.015 < x[256:].std() < 0.025
    np.testing.assert_array_equal(x, bf16_round(x))            # already bf16-exact
    np.testing.assert_array_equal(x, workload("tiny_512").prompt())  # seeded: reproducible
    wts = w1.weights(0)
    assert wts.wq.shape == (256, 256) and wts.wk.shape == (128, 256) and wts.wd.shape == (256, 1024)
    assert 0.018 < wts.wg.std() < 0.022 and np.all(wts.g1 == 1.0) and wts.bq is None
    assert w1.weights(0, qkv_bias=True, gains="uniform").bq.shape == (256,)


def test_batch_workload_lengths():
    w4 = workload(4)
    rng = np.random.default_rng(3)
    for _ in range(20):
        lens = synth.dirichlet_chunk_lengths(rng, 16, 2048)
        assert lens.sum() == 2048 and lens.min() >= 1 and len(lens) == 16
    lens = synth.dirichlet_chunk_lengths(rng, 4, 4)
    np.testing.assert_array_equal(lens, [1, 1, 1, 1])
    # a reduced copy of workload 4 (same recipe, small caches) so the test stays cheap
    small = synth.Workload("b", TINY, 1, 64, [1], n_requests=5, batch_seed=9, max_prior=40)
    reqs = small.batch()
    assert sum(r.rows.shape[0] for r in reqs) == 64
    for r in reqs:
        assert 0 <= r.prior_len <= 40 and r.prior_k.shape == (r.prior_len, 2, 64) == r.prior_v.shape
        assert r.rows.shape[1] == 256
    assert w4.n_requests == 16 and w4.max_prior == 12288 and w4.budget == 2048
