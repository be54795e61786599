#!/usr/bin/env python3
"""Time to first token of one multimodal request on one MI355X as a function of the embedding batch size C of
Algorithm 1 (section 3.2; the paper's 'embedding batch size' study, section 4.3): the stand-in encoder runs on its own
stream in batches of at least C multimodal tokens while the language model prefills what has become schedulable.

C = the whole request reproduces the behaviour of systems that encode everything before prefill starts (no overlap).
Prints one JSON line per C.  Synthetic data: the benchmark prompt of bench.py (6 images of 1024 embedding rows,
interleaved with text) through 28 7B-shaped layers (the 4 synthetic ones reused cyclically); the encoder is a stand-in
of configurable cost.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--encoder-gflop-per-token", type=float, default=4.0,
                    help="cost of the stand-in encoder per multimodal token")
    ap.add_argument("--layers", type=int, default=28,
                    help="decoder layers the prefill runs through (the 4 synthetic layers are reused cyclically: same "
                         "cost as distinct weights, 1/7 of the memory)")
    ap.add_argument("--budget", type=int, default=2048)
    ap.add_argument("--vocab", type=int, default=152064,
                    help="rows of the vocabulary matrix of the first-token head (final RMSNorm + projection of the last prompt row, "
                         "then the arg max, all inside the measured time); 0 stops the clock when the prefill is complete")
    ap.add_argument("--repeats", type=int, default=5)
    ap.add_argument("--batch-sizes", type=int, nargs="*", default=[256, 512, 1024, 2048, 4096, 1 << 30])
    args = ap.parse_args()

    import torch
    import synth
    from paper_2509_24381_amd import pipeline, runner

    assert torch.cuda.is_available(), "pipeline_bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = synth.workload(3)
    weights = [wl.weights(l) for l in range(wl.n_layers)]
    stack = runner.LayerStack(wl.shape, weights, max_tokens=args.budget, max_requests=1, max_pos=wl.n_tokens)
    del weights
    stack.layers = [stack.layers[l % wl.n_layers] for l in range(args.layers)]
    segments = [(kind == "image", n) for kind, n in wl.segments]
    rows = runner.to_device_bf16(wl.prompt())
    enc = pipeline.StubEncoder(args.encoder_gflop_per_token)
    head = None
    if args.vocab > 0:
        gen = torch.Generator(device="cuda").manual_seed(7)
        head = (torch.ones(wl.shape.hidden, device="cuda", dtype=torch.bfloat16),
                (torch.randn(args.vocab, wl.shape.hidden, device="cuda", generator=gen) * 0.02).to(torch.bfloat16))
    n_mm = sum(n for mm, n in segments if mm)
    for c in args.batch_sizes:
        times, enc_times, res = [], [], None
        for rep in range(args.repeats + 1):
            res, kv, out = pipeline.run_intra_request_pipeline(stack, segments, rows, min_tokens=c, token_budget=args.budget,
                                                               encoder=enc, head=head)
            if rep:                      # the first repetition warms up
                times.append(res.ttft_ms)
                enc_times.append(res.encode_ms)
            del kv, out
        times.sort()
        print(json.dumps({"metric": "time to first token of one request (" + ("first token on the host" if head else "prefill complete")
                                    + "), intra-request pipeline",
                          "embedding_batch_size": "whole request" if c >= n_mm else c,
                          "ttft_ms_median": times[len(times) // 2], "ttft_ms_min": times[0],
                          "encode_done_ms_median": sorted(enc_times)[len(enc_times) // 2],
                          "encode_batches": res.n_encode_batches, "prefill_rounds": res.n_rounds,
                          "prompt_tokens": wl.n_tokens, "multimodal_tokens": n_mm, "layers": args.layers,
                          "token_budget": args.budget, "encoder_gflop_per_token": args.encoder_gflop_per_token,
                          "vocab": args.vocab, "first_token": res.first_token}), flush=True)


if __name__ == "__main__":
    main()
