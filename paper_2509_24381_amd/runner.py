"""Convenience driver over the binding: uploads numpy inputs, runs chunk schedules, brings results back.

Used by the tests, the smoke check and the benchmark.  It holds no arithmetic: numpy arrays are converted to
bf16 device tensors (the inputs are already bf16-exact), the library is called, results are copied back.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from .binding import KVPool, Context, KVCache, LayerConfig, PackedWeights


def to_device_bf16(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device="cuda", dtype=torch.bfloat16)


def to_numpy_f32(t) -> np.ndarray:
    import torch
    return t.to(dtype=torch.float32).cpu().numpy()


def config_for(shape, *, qkv_bias=False, max_tokens=4096, max_requests=64, max_pos=32768) -> LayerConfig:
    return LayerConfig(hidden=shape.hidden, n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads,
                       head_dim=shape.head_dim, mlp_inter=shape.mlp_inter, rms_eps=shape.rms_eps,
                       rope_theta=shape.rope_theta, qkv_bias=qkv_bias, max_tokens_per_call=max_tokens,
                       max_requests=max_requests, max_pos=max_pos)


def pack_layer(ctx: Context, w) -> PackedWeights:
    """`w` carries torch-layout float32 (bf16-exact) arrays g1, wq, wk, wv, wo, g2, wg, wu, wd and optional bq, bk, bv."""
    import torch
    w_qkv = to_device_bf16(np.concatenate([w.wq, w.wk, w.wv], axis=0))
    w_gu = to_device_bf16(np.concatenate([w.wg, w.wu], axis=0))
    b = None
    if getattr(w, "bq", None) is not None:
        b = to_device_bf16(np.concatenate([w.bq, w.bk, w.bv], axis=0))
    packed = ctx.pack_weights(to_device_bf16(w.g1), w_qkv, to_device_bf16(w.wo), to_device_bf16(w.g2), w_gu,
                              to_device_bf16(w.wd), b_qkv=b)
    torch.cuda.synchronize()  # the torch-layout temporaries may be freed after this
    return packed


class LayerStack:
    """L decoder layers of one shape on the GPU, plus a workspace sized for the token budget."""

    def __init__(self, shape, layer_weights: Sequence, *, max_tokens: int, max_requests: int = 64,
                 max_pos: int = 32768, qkv_bias: bool = False, fp8_visible_tokens: int = 0):
        self.shape = shape
        self.ctx = Context(config_for(shape, qkv_bias=qkv_bias, max_tokens=max_tokens, max_requests=max_requests,
                                      max_pos=max_pos))
        self.layers: List[PackedWeights] = [pack_layer(self.ctx, w) for w in layer_weights]
        # (fp8_visible_tokens: room for the bf16 expansion that calls on 8-bit caches need, see Context.workspace)
        self.ws = self.ctx.workspace(max_tokens, max_requests, fp8_visible_tokens)

    @property
    def n_layers(self) -> int:
        return len(self.layers)

    def new_cache(self, capacity: int) -> KVCache:
        return self.ctx.kv_alloc(self.n_layers, capacity)

    def new_cache_fp8(self, capacity: int, k_scale: float = 1.0, v_scale: float = 1.0) -> KVCache:
        return self.ctx.kv_alloc_fp8(self.n_layers, capacity, k_scale, v_scale)

    def new_pool(self, n_pages: int, fp8: bool = False) -> KVPool:
        """A pool of KV pages (64 tokens of one layer each; fp8: of E4M3 bytes); `pool.new_cache(stack.n_layers)` gives
        growable caches."""
        return KVPool(self.ctx, n_pages, fp8=fp8)

    def prefill_prompt(self, x_dev, chunks: Sequence[Tuple[int, int]], kv: KVCache, keep_layer_outputs: bool = False):
        """Runs one request's prompt chunk by chunk through all layers: one rs_prefill_model_batch call per chunk, or -
        when every layer's output is wanted - one rs_prefill_chunk call per chunk and layer.

        x_dev: bf16 [N, H] device tensor.  Returns the final layer's output [N, H] (and, if asked, every layer's).
        """
        import torch
        n = x_dev.shape[0]
        if not keep_layer_outputs:   # all layers of a chunk in one call (the same bits as layer by layer)
            last = torch.empty_like(x_dev)
            for a, b in chunks:
                self.ctx.prefill_model_batch(self.layers, [kv], [b - a], x_dev[a:b], last[a:b], self.ws)
            return last
        outs = [torch.empty_like(x_dev) for _ in range(self.n_layers)] if keep_layer_outputs else None
        last = torch.empty_like(x_dev)
        scratch = torch.empty_like(x_dev)
        for a, b in chunks:
            cur = x_dev[a:b]
            for l, pw in enumerate(self.layers):
                if keep_layer_outputs:
                    dst = outs[l][a:b]
                else:
                    dst = last[a:b] if l == self.n_layers - 1 else scratch[a:b]
                self.ctx.prefill_chunk(pw, l, kv, cur, dst, self.ws)
                cur = dst
        if keep_layer_outputs:
            return outs[-1], outs
        return last

    def prefill_batch(self, layer: int, kvs: Sequence[KVCache], chunk_lens: Sequence[int], x_dev, y_dev=None):
        import torch
        if y_dev is None:
            y_dev = torch.empty_like(x_dev)
        return self.ctx.prefill_batch(self.layers[layer], layer, kvs, chunk_lens, x_dev, y_dev, self.ws)


def run_scheduled_round(stack: LayerStack, entries, embeddings, kvs, outputs) -> int:
    """BatchExecute(S) of Algorithm 2 for one scheduling round.

    entries: what Scheduler.next_round() returned; embeddings / kvs / outputs: dicts keyed by request id holding the
    request's bf16 [p, H] embedding tensor (the tracker's cache), its KVCache and the [p, H] tensor that receives the last
    layer's output.  Gathers the scheduled rows into the packed micro-batch input, runs every layer with
    rs_prefill_model_batch, scatters the result.  Returns the number of tokens run.
    """
    import torch
    live = [(rid, first, n) for rid, first, n, _ in entries if n > 0]
    if not live:
        return 0
    x = torch.cat([embeddings[rid][first: first + n] for rid, first, n in live], dim=0)
    lens = [n for _, _, n in live]
    batch_kvs = [kvs[rid] for rid, _, _ in live]
    stack.ctx.prefill_model_batch(stack.layers, batch_kvs, lens, x, x, stack.ws)   # all layers, in place
    off = 0
    for rid, first, n in live:
        outputs[rid][first: first + n] = x[off: off + n]
        off += n
    return off
