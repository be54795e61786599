"""Times one decoder-layer call for short chunks on long caches (7B shape), with and without split key ranges.

RServe schedules whatever tokens have become schedulable (Algorithm 2), so late in a long multimodal prompt a round is
often a few hundred rows on top of a cache of tens of thousands.  Such a call has fewer attention blocks than compute
units; the library then cuts each block's key range into parts (see AttnPartial in csrc/attention.h).  This script
measures what that is worth:  python short_chunk_bench.py  prints one markdown table row per (chunk, cache) pair.
With  --case ROWS,CACHED  (repeatable) only those pairs run, and only in the default configuration: the form a kernel
trace of short calls is taken with.
Synthetic inputs (N(0,1) cache content and rows, N(0, 0.02) weights); inputs resident; HIP events on the call's stream.
"""
import argparse
import os

import torch

import synth
from paper_2509_24381_amd import runner


def time_case(shape, w, t_rows, prior, split_env, reps):
    if split_env is None:
        os.environ.pop("RS_ATTN_SPLIT", None)
    else:
        os.environ["RS_ATTN_SPLIT"] = split_env          # read once, when the context is created
    stack = runner.LayerStack(shape, [w], max_tokens=t_rows, max_requests=1, max_pos=prior + t_rows)
    kv = stack.new_cache(prior + t_rows)
    g = torch.Generator(device="cuda").manual_seed(20250924)
    k = torch.randn(prior, shape.n_kv_heads, shape.head_dim, device="cuda", generator=g).to(torch.bfloat16)
    v = torch.randn(prior, shape.n_kv_heads, shape.head_dim, device="cuda", generator=g).to(torch.bfloat16)
    kv.import_(0, k, v)
    x = torch.randn(t_rows, shape.hidden, device="cuda", generator=g).to(torch.bfloat16)
    y = torch.empty_like(x)

    def call():
        kv.truncate(0, prior)
        stack.prefill_batch(0, [kv], [t_rows], x, y)

    for _ in range(3):
        call()
    torch.cuda.synchronize()
    stack.ctx.profile_enable("attention", reps)
    for _ in range(reps):
        call()
    torch.cuda.synchronize()
    ms, n = stack.ctx.profile_read()
    stack.ctx.profile_enable(None)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        call()
    e1.record()
    torch.cuda.synchronize()
    return ms / n * 1e3, e0.elapsed_time(e1) / reps * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--case", action="append", default=[], metavar="ROWS,CACHED",
                    help="run only this (chunk rows, cached tokens) pair, default configuration only; repeatable")
    args = ap.parse_args()
    cases = [tuple(int(v) for v in c.split(",")) for c in args.case]
    if any(len(c) != 2 or c[0] < 1 or c[1] < 0 for c in cases):
        ap.error("--case takes ROWS,CACHED with ROWS >= 1 and CACHED >= 0")
    shape = synth.L7B
    w = synth.layer_weights(shape, 1)
    print("| chunk rows | cached tokens | attention us, whole key range per block | attention us, split | layer call us, whole | layer call us, split |")
    print("|---:|---:|---:|---:|---:|---:|")
    for t_rows, prior in cases:
        a1, c1 = time_case(shape, w, t_rows, prior, None, args.reps)
        print(f"| {t_rows} | {prior} | - | {a1:.0f} | - | {c1:.0f} |", flush=True)
    if cases:
        return
    for t_rows, prior in ((64, 2048), (512, 1536), (64, 8192), (256, 8192), (256, 32768), (256, 131072), (512, 16384), (1024, 8192), (2048, 6144)):
        a0, c0 = time_case(shape, w, t_rows, prior, "1", args.reps)
        a1, c1 = time_case(shape, w, t_rows, prior, None, args.reps)
        print(f"| {t_rows} | {prior} | {a0:.0f} | {a1:.0f} | {c0:.0f} | {c1:.0f} |", flush=True)


if __name__ == "__main__":
    main()
