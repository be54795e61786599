"""Seeded, synthetic LMM-shaped workloads (shapes, value distributions, chunk schedules).

Everything here is input preparation: drawing numbers from numpy's PCG64
generator, rounding them once to bf16 (round-to-nearest-even) and laying out
prompts as image-embedding / text-embedding row segments.  The same arrays are
handed to the CPU oracle (promoted to fp64) and to the HIP path (as bf16 bit
patterns), so a comparison of the two measures arithmetic, not input
quantisation.

The five named workloads mirror the paper's workload statistics (section 4.1.2:
prompts of roughly 8k-12k tokens, most of them multimodal; section 4.3: 1024
tokens per high-quality multimodal item) on the Qwen2.5-VL-sized decoder shapes
the paper evaluates (section 4.1.1).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20250924


# --------------------------------------------------------------------------- bf16 helpers
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 values (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round a float array to the nearest bf16 value, returned as float32."""
    return bits_to_f32(bf16_bits(x))


# --------------------------------------------------------------------------- shapes
@dataclass(frozen=True)
class LayerShape:
    name: str
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_inter: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_dim(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def linear_flops_per_token(self) -> int:
        h, i = self.hidden, self.mlp_inter
        return 2 * (h * self.qkv_dim + self.q_dim * h + 3 * h * i)

    def attn_flops(self, t: int, p: int) -> int:
        """Causal-exact attention FLOPs of a chunk of t rows against a prefix of p tokens."""
        return 4 * self.n_q_heads * self.head_dim * (t * p + t * (t + 1) // 2)

    def weight_bytes(self) -> int:
        h, i = self.hidden, self.mlp_inter
        return 2 * (h * self.qkv_dim + self.q_dim * h + 3 * h * i + 2 * h)


TINY = LayerShape("tiny", 256, 4, 2, 64, 1024)
L7B = LayerShape("7b", 3584, 28, 4, 128, 18944)
L72B = LayerShape("72b", 8192, 64, 8, 128, 29568)


# --------------------------------------------------------------------------- weights
@dataclass
class LayerWeights:
    """One decoder layer's parameters, torch layout ([out, in]), float32 holding bf16-exact values."""
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

    def has_bias(self) -> bool:
        return self.bq is not None


def _normal_bf16(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return bf16_round(a)


def layer_weights(shape: LayerShape, seed: int, *, qkv_bias: bool = False,
                  gains: str = "ones", std: float = 0.02) -> LayerWeights:
    """Draw one layer's weights: matrices ~N(0, std) (std, not variance); norm gains 1 or U(0.5,1.5)."""
    rng = np.random.default_rng(seed)
    h, i = shape.hidden, shape.mlp_inter
    wq = _normal_bf16(rng, (shape.q_dim, h), std)
    wk = _normal_bf16(rng, (shape.kv_dim, h), std)
    wv = _normal_bf16(rng, (shape.kv_dim, h), std)
    wo = _normal_bf16(rng, (h, shape.q_dim), std)
    wg = _normal_bf16(rng, (i, h), std)
    wu = _normal_bf16(rng, (i, h), std)
    wd = _normal_bf16(rng, (h, i), std)
    if gains == "ones":
        g1 = np.ones(h, dtype=np.float32)
        g2 = np.ones(h, dtype=np.float32)
    elif gains == "uniform":
        g1 = bf16_round(rng.uniform(0.5, 1.5, h).astype(np.float32))
        g2 = bf16_round(rng.uniform(0.5, 1.5, h).astype(np.float32))
    else:
        raise ValueError(gains)
    w = LayerWeights(g1=g1, wq=wq, wk=wk, wv=wv, wo=wo, g2=g2, wg=wg, wu=wu, wd=wd)
    if qkv_bias:
        w.bq = _normal_bf16(rng, (shape.q_dim,), std)
        w.bk = _normal_bf16(rng, (shape.kv_dim,), std)
        w.bv = _normal_bf16(rng, (shape.kv_dim,), std)
    return w


# --------------------------------------------------------------------------- prompts
Segment = Tuple[str, int]  # ("image" | "text", n_rows)

IMAGE_STD = 1.0   # multimodal-encoder output rows
TEXT_STD = 0.02   # token-embedding rows


def prompt_rows(segments: Sequence[Segment], hidden: int, seed: int) -> np.ndarray:
    """Rows of one request's input embeddings: image rows ~N(0,1), text rows ~N(0,0.02), bf16-exact."""
    rng = np.random.default_rng(seed)
    parts = []
    for kind, n in segments:
        if kind == "image":
            parts.append(_normal_bf16(rng, (n, hidden), IMAGE_STD))
        elif kind == "text":
            parts.append(_normal_bf16(rng, (n, hidden), TEXT_STD))
        else:
            raise ValueError(kind)
    if not parts:
        return np.zeros((0, hidden), dtype=np.float32)
    return np.concatenate(parts, axis=0)


def chunk_schedule(n_tokens: int, budget: int) -> List[Tuple[int, int]]:
    """[start, end) row ranges of consecutive chunks of at most `budget` rows."""
    return [(s, min(s + budget, n_tokens)) for s in range(0, n_tokens, budget)]


def dirichlet_chunk_lengths(rng: np.random.Generator, n_requests: int, budget: int) -> np.ndarray:
    """Chunk lengths >= 1 that sum to `budget`: 1 + largest-remainder rounding of (budget-R)*w, w~Dirichlet(1)."""
    w = rng.dirichlet(np.ones(n_requests))
    spare = budget - n_requests
    raw = spare * w
    base = np.floor(raw).astype(np.int64)
    short = spare - int(base.sum())
    order = np.argsort(-(raw - base), kind="stable")
    base[order[:short]] += 1
    return base + 1


@dataclass
class BatchRequest:
    """One request's contribution to a multi-request micro-batch."""
    prior_len: int
    prior_k: np.ndarray   # [prior_len, Hkv, d]  post-RoPE keys already cached (bf16-exact float32)
    prior_v: np.ndarray   # [prior_len, Hkv, d]
    rows: np.ndarray      # [T_i, hidden] this round's chunk


@dataclass
class Workload:
    name: str
    shape: LayerShape
    n_layers: int
    budget: int
    weight_seeds: List[int]
    # single-request prompt (workloads 1, 2, 3, 5)
    segments: List[Segment] = field(default_factory=list)
    input_seed: int = 0
    # multi-request micro-batch (workload 4)
    n_requests: int = 0
    batch_seed: int = 0
    max_prior: int = 0

    @property
    def n_tokens(self) -> int:
        return sum(n for _, n in self.segments)

    def weights(self, layer: int = 0, **kw) -> LayerWeights:
        return layer_weights(self.shape, self.weight_seeds[layer], **kw)

    def prompt(self) -> np.ndarray:
        return prompt_rows(self.segments, self.shape.hidden, self.input_seed)

    def chunks(self) -> List[Tuple[int, int]]:
        return chunk_schedule(self.n_tokens, self.budget)

    def text_row_mask(self) -> np.ndarray:
        """True for the prompt rows that are text-token embeddings (the small-magnitude rows)."""
        return np.concatenate([np.full(n, kind == "text") for kind, n in self.segments])

    def batch(self) -> List[BatchRequest]:
        """Workload 4: 16 requests, prior cache lengths U{0..max_prior}, chunk lengths Dirichlet(1)."""
        assert self.n_requests > 0
        rng = np.random.default_rng(self.batch_seed)
        sh = self.shape
        prior = rng.integers(0, self.max_prior + 1, size=self.n_requests)
        lens = dirichlet_chunk_lengths(rng, self.n_requests, self.budget)
        out = []
        for p, t in zip(prior.tolist(), lens.tolist()):
            pk = _normal_bf16(rng, (p, sh.n_kv_heads, sh.head_dim), 1.0)
            pv = _normal_bf16(rng, (p, sh.n_kv_heads, sh.head_dim), 1.0)
            n_img = t // 2
            img = _normal_bf16(rng, (n_img, sh.hidden), IMAGE_STD)
            txt = _normal_bf16(rng, (t - n_img, sh.hidden), TEXT_STD)
            out.append(BatchRequest(p, pk, pv, np.concatenate([img, txt], axis=0)))
        return out


WORKLOAD_NAMES = ("tiny_512", "7b_2048_b512", "7b_x4_8192_b2048", "7b_batch16_b2048", "72b_32768_b4096")


def workload(name_or_index) -> Workload:
    """The five benchmark/parity workloads (index 1..5 or name)."""
    if isinstance(name_or_index, int):
        idx = name_or_index
    else:
        idx = WORKLOAD_NAMES.index(name_or_index) + 1
    seed0 = BASE_SEED + 1000 * idx
    if idx == 1:
        return Workload(WORKLOAD_NAMES[0], TINY, 1, 128, [seed0],
                        segments=[("image", 256), ("text", 256)], input_seed=seed0 + 500)
    if idx == 2:
        return Workload(WORKLOAD_NAMES[1], L7B, 1, 512, [seed0],
                        segments=[("image", 1280), ("text", 768)], input_seed=seed0 + 500)
    if idx == 3:
        segs: List[Segment] = []
        for _ in range(5):
            segs += [("image", 1024), ("text", 256)]
        segs += [("image", 1024), ("text", 768)]
        return Workload(WORKLOAD_NAMES[2], L7B, 4, 2048, [seed0 + l for l in range(4)],
                        segments=segs, input_seed=seed0 + 500)
    if idx == 4:
        return Workload(WORKLOAD_NAMES[3], L7B, 1, 2048, [seed0], n_requests=16,
                        batch_seed=seed0 + 700, max_prior=12288)
    if idx == 5:
        segs = [("image", 256)] * 120 + [("text", 2048)]
        return Workload(WORKLOAD_NAMES[4], L72B, 1, 4096, [seed0],
                        segments=segs, input_seed=seed0 + 500)
    raise ValueError(name_or_index)
