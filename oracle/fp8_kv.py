"""An 8-bit KV cache for chunked prefill, stated plainly (TEST INFRASTRUCTURE ONLY).

The paper configures every system it measures for the largest KV memory that fits (section 4.1.3) and serves
prompts of tens of thousands of multimodal tokens (section 2.1.1, section 4.1.2); it says nothing about the
storage type of the cache.  This module states the variant in which the cache holds one byte per element:

    code  = e4m3( fl32( bf16(x) * fl32(1 / scale) ) )      stored
    value = bf16( fl32( decode(code) * scale ) )           what attention reads

with one scale for all keys and one for all values of a cache.  `e4m3` is the OCP 8-bit floating-point format
E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, S.1111.111 is NaN, largest finite
value 448; exponent field 0 holds subnormals m/8 * 2^-6), rounding to the nearest representable value with ties
to the even mantissa and saturating at +-448.  Every token's K~ and V go through this on their way into the cache,
the tokens of the running chunk included, so the result does not depend on how the prompt is cut into chunks
(section 2.2.1's contract holds for the quantised model as it does for the exact one).

A quantised code is an integer decision, so it is taken in the precision the kernels hold the number in: the
bfloat16 value of K~ or V, one fp32 multiplication, then the rounding above.  The encoder below is the definition
written out: among all finite codes pick the nearest value, on a tie the one with the even mantissa.  It never
looks at bit fields of its input.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from .decoder_layer import ChunkedPrefill, LayerParams, _mlp_residual, _project_qkv, _softmax_rows, rmsnorm, rope

F64 = np.float64
E4M3_MAX = 448.0


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """The real number each E4M3 byte stands for, as float64 (NaN for 0x7f and 0xff)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c >= 128, -1.0, 1.0)
    e = (c >> 3) & 15
    m = c & 7
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(F64))
    subnormal = (m / 8.0) * 2.0 ** -6
    val = sign * np.where(e == 0, subnormal, normal)
    return np.where((e == 15) & (m == 7), np.nan, val)


def _finite_magnitudes() -> np.ndarray:
    """decode(0x00 .. 0x7e): the 127 non-negative finite values in increasing order (index = code)."""
    return e4m3_decode(np.arange(0x7F, dtype=np.uint8))


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 code of each number (ties to the even code, which has the even mantissa; |x| >= 448 gives +-448;
    NaN gives 0x7f; the sign of zero is kept)."""
    x = np.asarray(x, dtype=F64)
    mags = _finite_magnitudes()
    a = np.minimum(np.abs(np.where(np.isnan(x), 0.0, x)), E4M3_MAX)
    hi = np.clip(np.searchsorted(mags, a, side="left"), 0, len(mags) - 1)   # first code with value >= a
    lo = np.maximum(hi - 1, 0)
    d_hi = mags[hi] - a
    d_lo = a - mags[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.int64)
    code = code | np.where(np.signbit(x), 128, 0)
    return np.where(np.isnan(x), 0x7F, code).astype(np.uint8)


def _bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 (ties to even), returned as float32: a bfloat16 is an fp32 whose low 16 bits are zero."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    keep = (u >> 16) & 1
    r = ((u + 0x7FFF + keep) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32).reshape(f.shape)
    return np.where(np.isnan(f), f, out)


def kv_store(x: np.ndarray, scale: float) -> np.ndarray:
    """Codes the cache keeps for the values x (any real array) under `scale`."""
    inv = np.float32(1.0) / np.float32(scale)
    with np.errstate(over="ignore", invalid="ignore"):   # (infinities saturate, NaNs stay NaN: both are meant)
        return e4m3_encode((_bf16(x) * inv).astype(np.float32))


def kv_load(codes: np.ndarray, scale: float) -> np.ndarray:
    """Values attention reads back from the codes (float64 holding bfloat16 numbers)."""
    v = e4m3_decode(codes).astype(np.float32) * np.float32(scale)
    return _bf16(v).astype(F64)


class ChunkedPrefillFp8KV(ChunkedPrefill):
    """ChunkedPrefill whose cache holds E4M3 codes: every K~ and V row is replaced by kv_load(kv_store(row)) before
    anything reads it, the running chunk's own rows included.  `codes_k` / `codes_v` keep what the cache stores."""

    def __init__(self, params: LayerParams, k_scale: float = 1.0, v_scale: float = 1.0):
        super().__init__(params)
        self.k_scale = float(k_scale)
        self.v_scale = float(v_scale)
        hkv, d = params.n_kv_heads, params.head_dim
        self.codes_k = np.zeros((0, hkv, d), dtype=np.uint8)
        self.codes_v = np.zeros((0, hkv, d), dtype=np.uint8)

    def prefill_chunk(self, x_chunk: np.ndarray) -> np.ndarray:
        p = self.p
        x_chunk = np.asarray(x_chunk, dtype=F64)
        t = x_chunk.shape[0]
        if t == 0:
            return x_chunk.copy()
        prefix = self.length
        pos = prefix + np.arange(t)
        h = rmsnorm(x_chunk, p.g1, p.rms_eps)
        q, k_new, v_new = _project_qkv(h, p)
        q = rope(q, pos, p.rope_theta)
        k_new = rope(k_new, pos, p.rope_theta)
        ck, cv = kv_store(k_new, self.k_scale), kv_store(v_new, self.v_scale)
        self.codes_k = np.concatenate([self.codes_k, ck], axis=0)
        self.codes_v = np.concatenate([self.codes_v, cv], axis=0)
        self.k = np.concatenate([self.k, kv_load(ck, self.k_scale)], axis=0)
        self.v = np.concatenate([self.v, kv_load(cv, self.v_scale)], axis=0)
        n = prefix + t
        scale = 1.0 / np.sqrt(F64(p.head_dim))
        o = np.empty((t, p.n_q_heads, p.head_dim), dtype=F64)
        visible = np.arange(n)[None, :] <= pos[:, None]
        for hh in range(p.n_q_heads):
            c = hh // p.group
            s = (q[:, hh, :] @ self.k[:, c, :].T) * scale
            a = _softmax_rows(np.where(visible, s, -np.inf))
            o[:, hh, :] = a @ self.v[:, c, :]
        r = x_chunk + o.reshape(t, -1) @ p.wo.T
        return _mlp_residual(r, p)


def layer_forward_fp8kv(x: np.ndarray, p: LayerParams, k_scale: float = 1.0, v_scale: float = 1.0,
                        row_block: Optional[int] = None):
    """Whole-prompt form of the same model: (Y, codes_k, codes_v).  Keys and values of all tokens go through the
    cache's storage format; queries do not."""
    from .decoder_layer import causal_gqa_attention
    x = np.asarray(x, dtype=F64)
    n = x.shape[0]
    pos = np.arange(n)
    h = rmsnorm(x, p.g1, p.rms_eps)
    q, k, v = _project_qkv(h, p)
    q = rope(q, pos, p.rope_theta)
    k = rope(k, pos, p.rope_theta)
    ck, cv = kv_store(k, k_scale), kv_store(v, v_scale)
    kw = {} if row_block is None else {"row_block": row_block}
    o = causal_gqa_attention(q, kv_load(ck, k_scale), kv_load(cv, v_scale), **kw)
    r = x + o.reshape(n, p.n_q_heads * p.head_dim) @ p.wo.T
    return _mlp_residual(r, p), ck, cv
