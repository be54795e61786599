"""Plain fp64 definition of the decoder layer that chunked prefill runs (TEST INFRASTRUCTURE ONLY).

What is computed.  The paper (section 2.1.1, "LLM inference procedure"; section
2.2.1, "Chunked pipeline parallelism") states the contract of chunked prefill:
the prompt is split into chunks processed one after another, a chunk depends on
earlier chunks only through the KV cache they left behind, and the result is the
same as prefilling the whole prompt at once (section 6 says the system does not
change model behaviour).  Algorithm 2 (section 3.3) hands the language model a
micro-batch holding tokens of several requests under one token budget; requests
never interact (section 4.1.3 disables cross-request KV reuse).

The paper does not describe the inside of the layer; it names the model family
(Qwen2.5-VL, section 4.1.1).  The layer below is the pre-norm decoder block of
that family with 1-D rotary positions:

    h   = rmsnorm(X; g1)                     q,k,v = h Wq^T (+bq), h Wk^T (+bk), h Wv^T (+bv)
    q~,k~ = rope(q), rope(k) at the token's absolute position
    o   = causal GQA softmax(q~ k~^T / sqrt(d)) v
    r   = X + o Wo^T
    Y   = r + ( silu(h2 Wg^T) * (h2 Wu^T) ) Wd^T,    h2 = rmsnorm(r; g2)
    cache <- (k~, v) appended in token order

Because the method is exact, `layer_forward` is that definition written out for
a whole prompt.  `ChunkedPrefill` is the same computation organised the way the
method runs it (chunk by chunk against a growing cache) and is written
separately so that "chunked == unchunked" is a real test.  `prefill_batch` is
independent per-request application.

All arithmetic is float64 with no intermediate rounding.  Library primitives used
as steps: numpy matmul, exp, sqrt, cos, sin.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


@dataclass
class LayerParams:
    """fp64 copy of one layer's parameters (torch layout: [out_features, in_features])."""
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_inter: int
    rms_eps: float
    rope_theta: float
    g1: np.ndarray
    wq: np.ndarray
    wk: np.ndarray
    wv: np.ndarray
    wo: np.ndarray
    g2: np.ndarray
    wg: np.ndarray
    wu: np.ndarray
    wd: np.ndarray
    bq: Optional[np.ndarray] = None
    bk: Optional[np.ndarray] = None
    bv: Optional[np.ndarray] = None

    @classmethod
    def from_arrays(cls, shape, weights) -> "LayerParams":
        """Promote any (shape, weights) pair of attribute-bearing objects to fp64."""
        def f(name):
            a = getattr(weights, name, None)
            return None if a is None else np.asarray(a, dtype=F64)
        return cls(hidden=int(shape.hidden), n_q_heads=int(shape.n_q_heads),
                   n_kv_heads=int(shape.n_kv_heads), head_dim=int(shape.head_dim),
                   mlp_inter=int(shape.mlp_inter), rms_eps=float(shape.rms_eps),
                   rope_theta=float(shape.rope_theta),
                   g1=f("g1"), wq=f("wq"), wk=f("wk"), wv=f("wv"), wo=f("wo"),
                   g2=f("g2"), wg=f("wg"), wu=f("wu"), wd=f("wd"),
                   bq=f("bq"), bk=f("bk"), bv=f("bv"))

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


# --------------------------------------------------------------------------- elementary pieces
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise x * g / sqrt(mean(x^2) + eps); eps sits inside the square root, no mean subtraction."""
    x = np.asarray(x, dtype=F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=F64)


def rope_angles(positions: np.ndarray, head_dim: int, theta: float) -> np.ndarray:
    """phi[n, j] = pos_n * theta^(-2j/d), j < d/2 (1-D rotary embedding)."""
    j = np.arange(head_dim // 2, dtype=F64)
    inv_freq = theta ** (-2.0 * j / head_dim)
    return np.asarray(positions, dtype=F64)[:, None] * inv_freq[None, :]


def mrope_angles(positions3: np.ndarray, head_dim: int, theta: float, sections: Sequence[int]) -> np.ndarray:
    """Three-axis rotary angles (the M-RoPE of the model family the paper serves; not in the paper's own text):
    positions3[n] = (temporal, height, width); the d/2 pairs are split into consecutive sections of sections[0],
    sections[1], sections[2] pairs, and pair j in section a turns by positions3[n, a] * theta^(-2j/d)."""
    assert sum(sections) == head_dim // 2
    positions3 = np.asarray(positions3, dtype=F64)
    phi = np.empty((positions3.shape[0], head_dim // 2), dtype=F64)
    j0 = 0
    for axis, count in enumerate(sections):
        for j in range(j0, j0 + count):
            phi[:, j] = positions3[:, axis] * theta ** (-2.0 * j / head_dim)
        j0 += count
    return phi


def rope(v: np.ndarray, positions: np.ndarray, theta: float, sections: Optional[Sequence[int]] = None) -> np.ndarray:
    """Rotate-half RoPE on v[n, head, d]: pairs (j, j + d/2) are rotated by phi[n, j].  positions is [n] (1-D RoPE)
    or, with `sections`, [n, 3] (three-axis RoPE, see mrope_angles)."""
    v = np.asarray(v, dtype=F64)
    d = v.shape[-1]
    half = d // 2
    phi = rope_angles(positions, d, theta) if sections is None else mrope_angles(positions, d, theta, sections)
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    out = np.empty_like(v)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


def silu(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=F64)
    return z / (1.0 + np.exp(-z))


def _softmax_rows(s: np.ndarray) -> np.ndarray:
    """softmax over the last axis: subtract the row max, exponentiate, divide by the row sum."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, *,
                         row_block: int = 1024, return_probs: bool = False):
    """Whole-sequence causal attention with grouped KV heads.

    q[N, Hq, d], k[N, Hkv, d], v[N, Hkv, d]; query head h uses KV head h // (Hq/Hkv);
    token n attends to tokens 0..n inclusive with scores q.k / sqrt(d).
    Query rows are evaluated in independent slabs of `row_block` rows only to bound
    memory; each row's softmax is taken over its full key range in one go.
    """
    n, hq, d = q.shape
    hkv = k.shape[1]
    g = hq // hkv
    scale = 1.0 / np.sqrt(F64(d))
    out = np.empty((n, hq, d), dtype=F64)
    probs = np.zeros((hq, n, n), dtype=F64) if return_probs else None
    key_idx = np.arange(n)
    for h in range(hq):
        c = h // g
        kh = k[:, c, :]
        vh = v[:, c, :]
        for a in range(0, n, row_block):
            b = min(a + row_block, n)
            s = (q[a:b, h, :] @ kh[:b].T) * scale              # [b-a, b]
            visible = key_idx[None, :b] <= np.arange(a, b)[:, None]
            s = np.where(visible, s, -np.inf)
            p = _softmax_rows(s)
            out[a:b, h, :] = p @ vh[:b]
            if return_probs:
                probs[h, a:b, :b] = p
    if return_probs:
        return out, probs
    return out


# --------------------------------------------------------------------------- whole-prompt definition
def _project_qkv(h: np.ndarray, p: LayerParams):
    q = h @ p.wq.T
    k = h @ p.wk.T
    v = h @ p.wv.T
    if p.bq is not None:
        q = q + p.bq
        k = k + p.bk
        v = v + p.bv
    n = h.shape[0]
    return (q.reshape(n, p.n_q_heads, p.head_dim),
            k.reshape(n, p.n_kv_heads, p.head_dim),
            v.reshape(n, p.n_kv_heads, p.head_dim))


def _mlp_residual(r: np.ndarray, p: LayerParams) -> np.ndarray:
    h2 = rmsnorm(r, p.g2, p.rms_eps)
    a = silu(h2 @ p.wg.T) * (h2 @ p.wu.T)
    return r + a @ p.wd.T


def layer_forward(x: np.ndarray, p: LayerParams, positions3: Optional[np.ndarray] = None,
                  sections: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Unchunked prefill of one request through one layer.

    x[N, hidden] -> (Y[N, hidden], K~[N, Hkv, d] post-RoPE, V[N, Hkv, d]); token n sits at position n, or - when
    positions3[N, 3] and sections are given - is rotated by its three-axis position (causal order stays n).
    """
    x = np.asarray(x, dtype=F64)
    n = x.shape[0]
    pos = np.arange(n) if positions3 is None else positions3
    h = rmsnorm(x, p.g1, p.rms_eps)
    q, k, v = _project_qkv(h, p)
    q = rope(q, pos, p.rope_theta, sections if positions3 is not None else None)
    k = rope(k, pos, p.rope_theta, sections if positions3 is not None else None)
    o = causal_gqa_attention(q, k, v)
    r = x + o.reshape(n, p.n_q_heads * p.head_dim) @ p.wo.T
    y = _mlp_residual(r, p)
    return y, k, v


def layer_forward_rows(x: np.ndarray, p: LayerParams, rows: Sequence[int], row_block: int = 512):
    """The same definition evaluated for selected output rows only.

    The K~/V cache is still produced for every token (a row's attention needs all earlier
    keys), but queries, attention, the output projection and the MLP are evaluated only for
    `rows` (any order, output in the same order).  Returns (Y[rows], K~[N], V[N]).  Used where the
    full layer is too slow to run whole.  As in `causal_gqa_attention`, the selected rows are
    taken in slabs of `row_block` only to bound memory and time: a slab's scores are formed
    against every key up to the slab's latest position, keys after a row's own position are
    set to -inf, and each row's softmax is taken over its full visible key range in one go.
    """
    x = np.asarray(x, dtype=F64)
    n = x.shape[0]
    rows = np.asarray(rows, dtype=np.int64)
    h = rmsnorm(x, p.g1, p.rms_eps)
    k = h @ p.wk.T
    v = h @ p.wv.T
    if p.bk is not None:
        k = k + p.bk
        v = v + p.bv
    k = rope(k.reshape(n, p.n_kv_heads, p.head_dim), np.arange(n), p.rope_theta)
    v = v.reshape(n, p.n_kv_heads, p.head_dim)
    qs = h[rows] @ p.wq.T
    if p.bq is not None:
        qs = qs + p.bq
    qs = rope(qs.reshape(len(rows), p.n_q_heads, p.head_dim), rows, p.rope_theta)
    scale = 1.0 / np.sqrt(F64(p.head_dim))
    o = np.empty((len(rows), p.n_q_heads, p.head_dim), dtype=F64)
    by_position = np.argsort(rows, kind="stable")     # slabs of neighbouring positions waste the fewest masked keys
    for a in range(0, len(rows), row_block):
        sel = by_position[a: a + row_block]
        pos = rows[sel]
        t_end = int(pos.max()) + 1
        visible = np.arange(t_end)[None, :] <= pos[:, None]
        for hh in range(p.n_q_heads):
            c = hh // p.group
            s = (qs[sel, hh, :] @ k[:t_end, c, :].T) * scale
            s = np.where(visible, s, -np.inf)
            o[sel, hh, :] = _softmax_rows(s) @ v[:t_end, c, :]
    r = x[rows] + o.reshape(len(rows), -1) @ p.wo.T
    return _mlp_residual(r, p), k, v


# --------------------------------------------------------------------------- chunked form
class ChunkedPrefill:
    """One request's prefill state for one layer: the post-RoPE K and the V of every token so far.

    `prefill_chunk` consumes the next T rows of the prompt (positions P..P+T-1 where P is the
    number of cached tokens), lets them attend to the whole cache plus, causally, to each other,
    and appends their K~/V.  This follows the statement of chunked prefill in section 2.2.1.
    """

    def __init__(self, params: LayerParams, prior_k: Optional[np.ndarray] = None,
                 prior_v: Optional[np.ndarray] = None):
        self.p = params
        hkv, d = params.n_kv_heads, params.head_dim
        self.k = np.zeros((0, hkv, d), dtype=F64) if prior_k is None else np.asarray(prior_k, dtype=F64).copy()
        self.v = np.zeros((0, hkv, d), dtype=F64) if prior_v is None else np.asarray(prior_v, dtype=F64).copy()
        assert self.k.shape == self.v.shape

    @property
    def length(self) -> int:
        return self.k.shape[0]

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
        # append first: the chunk's own keys are part of what its rows may see
        self.k = np.concatenate([self.k, k_new], axis=0)
        self.v = np.concatenate([self.v, v_new], axis=0)
        scale = 1.0 / np.sqrt(F64(p.head_dim))
        o = np.empty((t, p.n_q_heads, p.head_dim), dtype=F64)
        # in-chunk causal frame: row i of the chunk sees chunk keys 0..i; every prefix key is visible
        in_chunk_hidden = np.triu(np.ones((t, t), dtype=bool), k=1)
        for hh in range(p.n_q_heads):
            c = hh // p.group
            s_prefix = (q[:, hh, :] @ self.k[:prefix, c, :].T) * scale      # [t, prefix]
            s_chunk = (q[:, hh, :] @ k_new[:, c, :].T) * scale              # [t, t]
            s_chunk = np.where(in_chunk_hidden, -np.inf, s_chunk)
            a = _softmax_rows(np.concatenate([s_prefix, s_chunk], axis=1))
            o[:, hh, :] = a[:, :prefix] @ self.v[:prefix, c, :] + a[:, prefix:] @ v_new[:, c, :]
        r = x_chunk + o.reshape(t, -1) @ p.wo.T
        return _mlp_residual(r, p)


def prefill_batch(states: List[ChunkedPrefill], chunks: List[np.ndarray]) -> np.ndarray:
    """A multi-request micro-batch (Algorithm 2's set S): each request's rows go through its own state.

    `chunks[i]` holds request i's rows for this round (possibly zero rows); the result is the packed
    [sum T_i, hidden] output in request order.  Requests do not interact.
    """
    assert len(states) == len(chunks)
    if len({id(s) for s in states}) != len(states):
        raise ValueError("a request may appear only once in a micro-batch")
    outs = [st.prefill_chunk(c) for st, c in zip(states, chunks)]
    hidden = states[0].p.hidden if states else 0
    if not outs:
        return np.zeros((0, hidden), dtype=F64)
    return np.concatenate(outs, axis=0)


def first_token_logits(x_rows: np.ndarray, gain: np.ndarray, w_lm: np.ndarray, eps: float) -> np.ndarray:
    """Final RMSNorm and vocabulary projection of hidden-state rows: logits[r, v] = rmsnorm(x_r; gain) . w_lm[v].

    The paper's latency metric is the time to the first token (section 4.1.4); this is the step that turns the last
    prompt row's hidden state into that token's scores.  Same RMSNorm as inside the layers; w_lm in torch layout
    [vocab, hidden]."""
    return rmsnorm(x_rows, gain, eps) @ np.asarray(w_lm, dtype=F64).T


def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    """Relative Frobenius error ||got - want||_F / ||want||_F (0 when both are empty/zero)."""
    got = np.asarray(got, dtype=F64)
    want = np.asarray(want, dtype=F64)
    den = float(np.linalg.norm(want))
    num = float(np.linalg.norm(got - want))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
