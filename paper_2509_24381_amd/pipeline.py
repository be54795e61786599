"""Intra-request pipeline on one GPU (section 3.2, Algorithm 1): multimodal items are encoded in batches of at least C
tokens on one stream while the language model prefills, on another stream, whatever tokens have become schedulable.

The multimodal encoder is outside this library's scope.  `StubEncoder` stands in for it: a stack of plain bf16 matmuls
sized to a given cost per multimodal token (it runs through PyTorch, like any caller-side model would), after which the
item's embedding rows - synthetic, drawn beforehand - are copied into the request's embedding buffer, the tracker's
cache of section 3.1.  Everything on the prefill side goes through the library: `Scheduler` (rs_sched_*) decides each
round, `run_scheduled_round` runs it with rs_prefill_batch.
"""
from __future__ import annotations

import time
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

from .binding import Scheduler
from .runner import LayerStack, run_scheduled_round


class StubEncoder:
    """A timed stand-in for the vision encoder: `gflop_per_token` of bf16 matmul work per multimodal token."""

    def __init__(self, gflop_per_token: float, width: int = 1280, patches_per_token: int = 4):
        import torch
        self.width = width
        self.patches = patches_per_token
        self.w = (torch.randn(width, width, device="cuda") * 0.02).to(torch.bfloat16)
        per_matmul = 2.0 * patches_per_token * width * width / 1e9      # GFLOP per token per matmul
        self.n_matmuls = max(1, int(round(gflop_per_token / per_matmul)))

    def encode(self, n_tokens: int):
        """Enqueues the stand-in work for `n_tokens` multimodal tokens on the current stream."""
        import torch
        h = torch.empty(n_tokens * self.patches, self.width, device="cuda", dtype=torch.bfloat16).normal_()
        for _ in range(self.n_matmuls):
            h = torch.mm(h, self.w)
        return h


@dataclass
class PipelineResult:
    ttft_ms: float            # request arrival -> last prompt token prefilled; with a head: -> first output token on the host
    encode_ms: float          # arrival -> last encoder batch delivered
    n_rounds: int
    n_encode_batches: int
    round_tokens: List[int]
    first_token: int = -1     # arg max of the first-token logits (only with a head)


def run_intra_request_pipeline(stack: LayerStack, segments: Sequence[Tuple[bool, int]], rows_dev, *, min_tokens: int,
                               token_budget: int, encoder: StubEncoder, request_id: int = 1,
                               head=None) -> Tuple[PipelineResult, object, object]:
    """Serves ONE request: Algorithm 1 feeds the encoder on its own stream, Algorithm 2 (with a single request in the
    queue) prefills on the current stream whatever has become schedulable.  rows_dev holds the prompt's final embedding
    rows (text rows are valid from the start; a multimodal item's rows count as available only once the encoder batch
    that contains it has finished).  head = (final_norm_gain [H], w_lm [vocab, H]) bf16 device tensors: the time to first
    token then includes the final RMSNorm and vocabulary projection of the last prompt row (rs_lm_head) and the arg max.
    Returns timings, the request's KV cache and the last layer's output."""
    import torch
    sched = Scheduler(token_budget)
    sched.add_request(request_id, segments)
    seg_begin = [0]
    for _, n in segments:
        seg_begin.append(seg_begin[-1] + n)
    n_total = seg_begin[-1]
    # the tracker's embedding cache: text rows present, multimodal rows filled in by the encoder
    emb = torch.zeros_like(rows_dev)
    for k, (mm, n) in enumerate(segments):
        if not mm:
            emb[seg_begin[k]: seg_begin[k + 1]] = rows_dev[seg_begin[k]: seg_begin[k + 1]]
    kv = stack.new_cache(n_total)
    out = torch.empty_like(rows_dev)
    batches = sched.encoder_batches(request_id, min_tokens)
    enc_stream = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # ---- Algorithm 1: every Encode(buffer) call goes to the encoder stream up front (FCFS); an event marks its end
    pending = []
    with torch.cuda.stream(enc_stream):
        for first_seg, last_seg, _, n_tok in batches:
            encoder.encode(n_tok)
            for k in range(first_seg, last_seg + 1):
                if segments[k][0]:
                    emb[seg_begin[k]: seg_begin[k + 1]].copy_(rows_dev[seg_begin[k]: seg_begin[k + 1]], non_blocking=True)
            ev = torch.cuda.Event()
            ev.record(enc_stream)
            pending.append((ev, first_seg, last_seg))
    # ---- Algorithm 2 with one request: prefill whatever is schedulable, as soon as it is
    rounds, round_tokens = 0, []
    t_encode = None
    while sched.queue_length():
        while pending and pending[0][0].query():
            ev, first_seg, last_seg = pending.pop(0)
            main.wait_event(ev)
            for k in range(first_seg, last_seg + 1):
                if segments[k][0]:
                    sched.mark_ready(request_id, k)
            if not pending:
                t_encode = time.perf_counter()
        if sched.schedulable_tokens(request_id) == 0:
            if pending:
                pending[0][0].synchronize()      # nothing to prefill: wait for the encoder
            continue
        entries = sched.next_round()
        n = run_scheduled_round(stack, entries, {request_id: emb}, {request_id: kv}, {request_id: out})
        rounds += 1
        round_tokens.append(n)
    first_token = -1
    if head is not None:
        logits = stack.ctx.lm_head(head[0], head[1], out[n_total - 1: n_total])
        first_token = int(torch.argmax(logits[0]).item())      # (the copy to the host waits for the stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    res = PipelineResult(ttft_ms=(t1 - t0) * 1e3, encode_ms=((t_encode or t1) - t0) * 1e3, n_rounds=rounds,
                         n_encode_batches=len(batches), round_tokens=round_tokens, first_token=first_token)
    return res, kv, out
