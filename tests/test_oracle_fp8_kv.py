"""Pins for the oracle's 8-bit KV cache (oracle/fp8_kv.py): the E4M3 codec against the format's definition, a
library conversion, brute force and its invariants; the quantised layer against the exact one and against itself
under re-chunking."""
import math

import numpy as np
import pytest
import torch

from oracle import ChunkedPrefill, layer_forward, rel_fro
from oracle.fp8_kv import (ChunkedPrefillFp8KV, e4m3_decode, e4m3_encode, kv_load, kv_store, layer_forward_fp8kv)
from test_oracle_pins import small_params


def all_bf16_values():
    """Every bfloat16 bit pattern as float32 (65536 values, NaNs and infinities included)."""
    bits = (np.arange(1 << 16, dtype=np.uint32) << 16)
    return bits.view(np.float32)


# ------------------------------------------------------------------ decode
def test_decode_values_the_format_fixes():
    # OCP 8-bit floating point, E4M3: bias 7, no infinities, one NaN pattern per sign, subnormals at exponent field 0
    want = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125, 0x3F: 1.875,
            0x40: 2.0, 0x78: 256.0, 0x7E: 448.0, 0xB8: -1.0, 0xFE: -448.0, 0x81: -(2.0 ** -9)}
    for code, val in want.items():
        assert e4m3_decode(np.array([code], dtype=np.uint8))[0] == val, hex(code)
    d = e4m3_decode(np.arange(256, dtype=np.uint8))
    assert np.isnan(d[0x7F]) and np.isnan(d[0xFF]) and np.isnan(d).sum() == 2
    assert np.signbit(d[0x80]) and d[0x80] == 0.0
    assert np.all(np.diff(d[:0x7F]) > 0)                 # codes 0..0x7e increase strictly
    assert np.array_equal(d[0x80:0xFF], -d[0x00:0x7F])   # the sign bit only flips the sign


def test_decode_matches_library_float8():
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = e4m3_decode(codes.numpy())
    assert np.array_equal(np.isnan(lib), np.isnan(got))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], got[ok]) and np.array_equal(np.signbit(lib[ok]), np.signbit(got[ok]))


# ------------------------------------------------------------------ encode
def test_encode_round_trips_every_code():
    codes = np.arange(256, dtype=np.uint8)
    back = e4m3_encode(e4m3_decode(codes))
    want = codes.copy()
    want[0xFF] = 0x7F  # both NaN patterns encode to the positive one
    assert np.array_equal(back, want)


def test_encode_is_the_nearest_code_by_exhaustive_search():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 1, 4000), rng.normal(0, 100, 2000), rng.uniform(-2.0 ** -5, 2.0 ** -5, 2000),
                        rng.uniform(-460, 460, 1000)])
    finite = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    vals = e4m3_decode(finite)
    got = e4m3_decode(e4m3_encode(x))
    best = np.min(np.abs(vals[None, :] - x[:, None]), axis=1)
    assert np.array_equal(np.abs(got - x), best)


def test_encode_ties_go_to_the_even_mantissa_and_large_values_saturate():
    # midpoints between neighbours: 1 + 1/16 lies between 1.0 (mantissa 0) and 1.125 (mantissa 1)
    assert e4m3_encode(np.array([1.0625]))[0] == 0x38
    assert e4m3_encode(np.array([1.1875]))[0] == 0x3A          # between 1.125 (m=1) and 1.25 (m=2)
    assert e4m3_encode(np.array([1.9375]))[0] == 0x40          # between 1.875 (m=7) and 2.0 (m=0 of the next binade)
    assert e4m3_encode(np.array([2.0 ** -10]))[0] == 0x00      # half the smallest subnormal: tie to zero
    assert e4m3_encode(np.array([3 * 2.0 ** -10]))[0] == 0x02  # between subnormals 1 and 2
    assert e4m3_encode(np.array([-1.0625]))[0] == 0xB8
    assert e4m3_encode(np.array([np.nextafter(1.0625, 2.0)]))[0] == 0x39
    for big in (448.0, 449.0, 464.0, 480.0, 1e6, np.inf):
        assert e4m3_encode(np.array([big]))[0] == 0x7E and e4m3_encode(np.array([-big]))[0] == 0xFE
    assert e4m3_encode(np.array([np.nan]))[0] == 0x7F
    assert e4m3_encode(np.array([-0.0]))[0] == 0x80


def test_encode_matches_library_float8_on_every_bf16_value_in_range():
    x = all_bf16_values()
    inside = np.isfinite(x) & (np.abs(x) <= 448.0)   # (the library does not saturate: beyond the range it gives NaN)
    lib = torch.from_numpy(x[inside].copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(e4m3_encode(x[inside]), lib)


def test_encode_is_monotone_and_odd():
    x = np.sort(all_bf16_values()[np.isfinite(all_bf16_values())].astype(np.float64))
    v = e4m3_decode(e4m3_encode(x))
    assert np.all(np.diff(v) >= 0)
    assert np.array_equal(e4m3_decode(e4m3_encode(-x)), -v)


# ------------------------------------------------------------------ store / load
def test_store_and_load_follow_their_formula_on_hand_values():
    # scale 0.5: 0.3 -> bf16 0.30078125 -> * 2 = 0.6015625 -> nearest of {0.5625, 0.625} is 0.625 (0x32) -> * 0.5
    assert kv_store(np.array([0.3]), 0.5)[0] == 0x32
    assert kv_load(np.array([0x32], dtype=np.uint8), 0.5)[0] == 0.3125
    # the bf16 rounding comes first: 1.064 lies above the tie 1.0625 (it would go up to 1.125), but bf16(1.064) = 1.0625
    # is the tie itself and goes to the even mantissa, 1.0
    assert kv_store(np.array([1.064]), 1.0)[0] == 0x38 and e4m3_encode(np.array([1.064]))[0] == 0x39
    # relative error of a stored value: half a step of 2^-3 relative to the binade, i.e. at most 1/16 + bf16 rounding
    rng = np.random.default_rng(2)
    x = rng.normal(0, 2.0, 20000)
    x = x[np.abs(x) > 2.0 ** -6]
    y = kv_load(kv_store(x, 1.0), 1.0)
    assert np.max(np.abs(y - x) / np.abs(x)) <= 1.0 / 16.0 + 2.0 ** -8
    # load rounds to bfloat16: with a scale that has a full mantissa the product needs it
    s = float(np.float32(1.0 / 3.0))
    y = kv_load(np.arange(0x7F, dtype=np.uint8), s)
    as_f32 = y.astype(np.float32)
    assert np.array_equal(as_f32.view(np.uint32) & 0xFFFF, np.zeros(0x7F, dtype=np.uint32))
    assert np.max(np.abs(y[1:] / (e4m3_decode(np.arange(1, 0x7F, dtype=np.uint8)) * s) - 1.0)) <= 2.0 ** -8


# ------------------------------------------------------------------ the quantised layer
def test_quantised_chunked_equals_quantised_unchunked_bit_for_bit_in_the_codes():
    rng = np.random.default_rng(11)
    p = small_params(rng, bias=True)
    x = rng.normal(0, 1, (37, p.hidden))
    y_full, ck, cv = layer_forward_fp8kv(x, p, 0.25, 0.5)
    for cuts in ([37], [5, 1, 20, 11], [16, 16, 5]):
        st = ChunkedPrefillFp8KV(p, 0.25, 0.5)
        outs, a = [], 0
        for t in cuts:
            outs.append(st.prefill_chunk(x[a:a + t]))
            a += t
        assert np.array_equal(st.codes_k, ck) and np.array_equal(st.codes_v, cv)
        assert rel_fro(np.concatenate(outs), y_full) < 1e-12


def test_quantised_layer_reduces_to_the_exact_one_when_the_cache_holds_exact_values():
    # K~ and V that are E4M3 numbers already survive the cache untouched: the 8-bit layer then equals the plain one.
    # With Wk = Wv = 0 and biases that are E4M3 values, every k and v row is the bias (V) or its rotation (K~):
    # position 0 only, where the rotation is the identity.
    rng = np.random.default_rng(3)
    p = small_params(rng, bias=True)
    p.wk[:] = 0.0
    p.wv[:] = 0.0
    p.bk[:] = e4m3_decode(rng.integers(0x20, 0x50, p.bk.shape).astype(np.uint8))
    p.bv[:] = -e4m3_decode(rng.integers(0x20, 0x50, p.bv.shape).astype(np.uint8))
    x = rng.normal(0, 1, (1, p.hidden))
    y_q, ck, cv = layer_forward_fp8kv(x, p)
    y, k, v = layer_forward(x, p)
    assert np.array_equal(e4m3_decode(ck), k) and np.array_equal(e4m3_decode(cv), v)
    assert rel_fro(y_q, y) < 1e-13


def test_quantised_layer_differs_from_the_exact_one_by_the_storage_error_only():
    rng = np.random.default_rng(8)
    p = small_params(rng)
    x = rng.normal(0, 1, (48, p.hidden))
    y, k, v = layer_forward(x, p)
    y_q, ck, cv = layer_forward_fp8kv(x, p)
    # the stored values are within half an E4M3 step (plus the bf16 rounding) of the exact ones ...
    big = np.abs(k) > 2.0 ** -6
    assert np.max(np.abs(kv_load(ck, 1.0) - k)[big] / np.abs(k)[big]) <= 1.0 / 16.0 + 2.0 ** -8
    assert np.max(np.abs(kv_load(cv, 1.0) - v)) <= np.max(np.abs(v)) / 16.0 + 2.0 ** -10
    # ... so the layer output moves, by per cents on this tiny, attention-dominated layer (and not by nothing: the
    # cache is really used)
    e = rel_fro(y_q, y)
    assert 1e-4 < e < 0.15
    # feeding the dequantised cache to the exact attention by hand gives the quantised output: nothing else changed
    st = ChunkedPrefill(p)
    st_q = ChunkedPrefillFp8KV(p)
    y1 = st_q.prefill_chunk(x[:20])
    st2 = ChunkedPrefill(p, prior_k=st_q.k, prior_v=st_q.v)   # continue exactly on the quantised prefix
    y2_q = st_q.prefill_chunk(x[20:21])
    y2 = st2.prefill_chunk(x[20:21])
    # the one new row attends to 20 quantised rows plus itself (exact in st2, quantised in st_q): close, not equal
    assert 0 < rel_fro(y2_q, y2) < 0.1
    assert y1.shape == (20, p.hidden) and st.length == 0


@pytest.mark.parametrize("scale", [1.0, 0.125, 3.0])
def test_scale_moves_the_range(scale):
    x = np.array([448.0 * scale, 500.0 * scale, -1000.0 * scale, 0.25 * scale])
    c = kv_store(x, scale)
    assert list(c[:3]) == [0x7E, 0x7E, 0xFE]
    assert math.isclose(kv_load(c, scale)[3], 0.25 * scale, rel_tol=2.0 ** -8)


# ------------------------------------------------------------------ the pins above can fail
def _decode_bias_8(codes):
    return e4m3_decode(codes) / 2.0                      # the other common 8-bit layout's exponent bias


def _decode_no_subnormals(codes):
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    v = e4m3_decode(codes)
    m, e = c & 7, (c >> 3) & 15
    return np.where(e == 0, np.where(c >= 128, -1.0, 1.0) * (1.0 + m / 8.0) * 2.0 ** -7 * (m > 0), v)


def _decode_with_infinity(codes):
    c = np.asarray(codes, dtype=np.uint8)
    return np.where((c & 0x7F) == 0x78, np.where(c >= 128, -np.inf, np.inf), e4m3_decode(codes))


def _encode_truncating(x):
    import oracle.fp8_kv as m
    x = np.asarray(x, dtype=np.float64)
    mags = m._finite_magnitudes()
    a = np.minimum(np.abs(np.where(np.isnan(x), 0.0, x)), 448.0)
    lo = np.clip(np.searchsorted(mags, a, side="right") - 1, 0, len(mags) - 1)
    return np.where(np.isnan(x), 0x7F, lo | np.where(np.signbit(x), 128, 0)).astype(np.uint8)


def _encode_ties_away(x):
    x = np.asarray(x, dtype=np.float64)
    return e4m3_encode(np.where(np.isnan(x), x, x * (1.0 + 2.0 ** -30)))


def _encode_overflow_to_nan(x):
    x = np.asarray(x, dtype=np.float64)
    return np.where(np.abs(x) > 464.0, 0x7F, e4m3_encode(x)).astype(np.uint8)


def _encode_drops_sign_of_zero(x):
    c = e4m3_encode(x)
    return np.where(c == 0x80, 0x00, c).astype(np.uint8)


def _store_without_bf16_rounding(x, scale):
    inv = np.float32(1.0) / np.float32(scale)
    return e4m3_encode((np.asarray(x, dtype=np.float32) * inv).astype(np.float32))


def _store_multiplies_by_scale(x, scale):
    import oracle.fp8_kv as m
    return e4m3_encode((m._bf16(x) * np.float32(scale)).astype(np.float32))


def _load_without_bf16_rounding(codes, scale):
    return (e4m3_decode(codes).astype(np.float32) * np.float32(scale)).astype(np.float64)


FP8_MUTANTS = [("e4m3_decode", _decode_bias_8), ("e4m3_decode", _decode_no_subnormals), ("e4m3_decode", _decode_with_infinity),
               ("e4m3_encode", _encode_truncating), ("e4m3_encode", _encode_ties_away), ("e4m3_encode", _encode_overflow_to_nan),
               ("e4m3_encode", _encode_drops_sign_of_zero), ("kv_store", _store_without_bf16_rounding),
               ("kv_store", _store_multiplies_by_scale), ("kv_load", _load_without_bf16_rounding)]


@pytest.mark.parametrize("name,mutant", FP8_MUTANTS, ids=[f.__name__.lstrip("_") for _, f in FP8_MUTANTS])
def test_planted_mistake_in_the_codec_is_caught(monkeypatch, name, mutant):
    """Each plausible mistake, planted in the oracle module (and in this module's imported names), must trip a pin."""
    import sys
    import oracle.fp8_kv as m
    me = sys.modules[__name__]
    monkeypatch.setattr(m, name, mutant)
    monkeypatch.setattr(me, name, mutant)
    calls = [test_decode_values_the_format_fixes, test_decode_matches_library_float8, test_encode_round_trips_every_code,
             test_encode_is_the_nearest_code_by_exhaustive_search,
             test_encode_ties_go_to_the_even_mantissa_and_large_values_saturate,
             test_encode_matches_library_float8_on_every_bf16_value_in_range, test_encode_is_monotone_and_odd,
             test_store_and_load_follow_their_formula_on_hand_values, lambda: test_scale_moves_the_range(0.125)]
    caught = []
    for call in calls:
        try:
            call()
        except AssertionError:
            caught.append(call)
        except Exception:
            caught.append(call)
    assert caught, f"no pin noticed {mutant.__name__}"
