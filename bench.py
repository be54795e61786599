#!/usr/bin/env python3
"""Benchmark of the chunked-prefill decoder-layer path on one MI355X.

A step is one pass of the whole hot path over the benchmark workload: a synthetic 8192-token multi-image prompt
(6 images of 1024 embedding rows interleaved with text spans) prefilled in 4 chunks under a 2048-token budget through
4 stacked 7B-shaped decoder layers, i.e. 4 rs_prefill_model_batch calls of 4 layers each (16 layer passes) with the KV
prefix growing 0 -> 6144.
`value` = layer-tokens per second (tokens x layers / time), inputs and weights resident in HBM.
`--workload 1..5` times one of the other parity workloads the same way (4 = the 16-request ragged micro-batch through
rs_prefill_batch, 5 = the 72B-shaped layer over a 32768-token prompt); the default, 3, is the headline configuration.

Prints ONE JSON line (see README / DESIGN for the fields): metric, value, ms_per_step, roofline of the dominant
kernel (the fused gate/up + SwiGLU GEMM, timed live with HIP events on its own stream inside the timed region), the
attention step's TFLOP/s and KV-read GB/s (one extra sampled pass after the timed region), and the fp64 CPU oracle
timed on a bounded sample of the same workload.

Two side studies share the harness (they print their own tables / lines, not the benchmark line):
  --short-chunks   one 7B-shaped layer call for short chunks on long caches, with and without split key ranges
                   (what Algorithm 2 produces late in a long prompt); --case ROWS,CACHED restricts it to given pairs
  --ttft           time to first token of one multimodal request against the embedding batch size C of Algorithm 1
                   (section 3.2 / the embedding-batch-size study of section 4.3), stand-in encoder on a second stream
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0
# Bytes crossing the L2 / fabric boundary per gate/up GEMM launch at T=2048 on the 7B shape: FETCH_SIZE and WRITE_SIZE
# (KiB per dispatch) from the two rocprofv3 --pmc passes summarised, with their date and commands, in
# profiles/gate_up_gemm_7b_T2048_hbm_traffic_pmc.md, each scaled by what the same counter reads for a plain copy kernel
# of known size (--copy-calibration).  Algorithmic bytes of the same launch: 363.9e6.
GATE_UP_FETCH_KIB, GATE_UP_FETCH_SCALE = 421650.6, 2.0
GATE_UP_WRITE_KIB, GATE_UP_WRITE_SCALE = 75776.0, 1.0
GATE_UP_TRAFFIC_BYTES = (GATE_UP_FETCH_KIB * GATE_UP_FETCH_SCALE + GATE_UP_WRITE_KIB * GATE_UP_WRITE_SCALE) * 1024


def cpu_baseline(wl, w0, x, target_seconds: float):
    """The oracle as it stands, one layer over the first rows of the same prompt, on the host cores.

    A 512-row probe estimates the host's speed; the reported sample is then sized for about `target_seconds` of CPU
    work (at most the whole prompt through layer 0)."""
    from oracle import LayerParams, layer_forward
    threads = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        blas = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
        if blas:
            threads = max(blas)
    except Exception:
        pass
    p = LayerParams.from_arrays(wl.shape, w0)

    def flops(rows):
        return wl.shape.linear_flops_per_token() * rows + wl.shape.attn_flops(rows, 0)

    def run(rows):
        t0 = time.perf_counter()
        layer_forward(x[:rows], p)
        return time.perf_counter() - t0

    probe_rows = min(512, x.shape[0])
    rate = flops(probe_rows) / run(probe_rows)
    rows = probe_rows
    while rows < x.shape[0] and flops(min(2 * rows, x.shape[0])) / rate <= target_seconds:
        rows = min(2 * rows, x.shape[0])
    dt = run(rows)
    return {"value": rows / dt, "unit": "layer-tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"fp64 oracle layer_forward, layer 0, first {rows} rows of the same prompt (P=0), {dt:.2f} s, "
                      f"{flops(rows) / dt / 1e9:.1f} GFLOP/s"}


def short_chunk_case(shape, w, t_rows, prior, split_env, reps):
    """(attention us, whole layer call us) of one call of t_rows rows on `prior` cached tokens; split_env "1" forbids
    split key ranges, None leaves the choice to the library (the hook is read once, when the context is created)."""
    import torch
    from paper_2509_24381_amd import runner
    if split_env is None:
        os.environ.pop("RS_ATTN_SPLIT", None)
    else:
        os.environ["RS_ATTN_SPLIT"] = split_env
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


def short_chunks(args):
    """Markdown table: one row per (chunk rows, cached tokens) pair.  Synthetic inputs (N(0,1) cache content and rows,
    N(0, 0.02) weights), resident; HIP events on the call's stream."""
    import synth
    cases = [tuple(int(v) for v in c.split(",")) for c in args.case]
    if any(len(c) != 2 or c[0] < 1 or c[1] < 0 for c in cases):
        sys.exit("--case takes ROWS,CACHED with ROWS >= 1 and CACHED >= 0")
    shape = synth.L7B
    w = synth.layer_weights(shape, 1)
    print("| chunk rows | cached tokens | attention us, whole key range per block | attention us, split | layer call us, whole | layer call us, split |")
    print("|---:|---:|---:|---:|---:|---:|")
    for t_rows, prior in cases:   # given pairs: the default configuration only (the form a kernel trace is taken with)
        a1, c1 = short_chunk_case(shape, w, t_rows, prior, None, args.reps)
        print(f"| {t_rows} | {prior} | - | {a1:.0f} | - | {c1:.0f} |", flush=True)
    if cases:
        return
    for t_rows, prior in ((64, 2048), (512, 1536), (64, 8192), (256, 8192), (256, 32768), (256, 131072), (512, 16384), (1024, 8192), (2048, 6144)):
        a0, c0 = short_chunk_case(shape, w, t_rows, prior, "1", args.reps)
        a1, c1 = short_chunk_case(shape, w, t_rows, prior, None, args.reps)
        print(f"| {t_rows} | {prior} | {a0:.0f} | {a1:.0f} | {c0:.0f} | {c1:.0f} |", flush=True)


def ttft_study(args):
    """One JSON line per embedding batch size C: the benchmark prompt through `--layers` 7B-shaped layers (the 4 synthetic
    ones reused cyclically: same cost as distinct weights, 1/7 of the memory); C = the whole request reproduces systems
    that encode everything before the prefill starts (no overlap)."""
    import torch
    import synth
    from paper_2509_24381_amd import pipeline, runner
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=3, choices=[1, 2, 3, 4, 5],
                    help="which of the five synthetic workloads to time (default 3: the headline configuration)")
    ap.add_argument("--breakdown", action="store_true", help="also time every step of the layer (extra passes)")
    ap.add_argument("--paged", action="store_true", help="keep the KV caches in pages of 64 tokens taken from one pool")
    ap.add_argument("--fp8-kv", action="store_true",
                    help="keep the KV caches as E4M3 bytes (scale 1/8), expanded per call for attention")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU work the oracle baseline sample is sized for")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, run one plain 256 MiB elementwise copy kernel (torch.mul(a, 1, out=b)); "
                         "gives the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs a kernel of known traffic to scale by")
    side = ap.add_argument_group("side studies (print their own output instead of the benchmark line)")
    side.add_argument("--short-chunks", action="store_true", help="short chunks on long caches, 7B shape (markdown table)")
    side.add_argument("--reps", type=int, default=20, help="--short-chunks: timed repetitions per case")
    side.add_argument("--case", action="append", default=[], metavar="ROWS,CACHED",
                      help="--short-chunks: only this (chunk rows, cached tokens) pair, default configuration only; repeatable")
    side.add_argument("--ttft", action="store_true", help="time to first token against the embedding batch size C of Algorithm 1")
    side.add_argument("--encoder-gflop-per-token", type=float, default=4.0, help="--ttft: cost of the stand-in encoder per multimodal token")
    side.add_argument("--layers", type=int, default=28, help="--ttft: decoder layers the prefill runs through")
    side.add_argument("--budget", type=int, default=2048, help="--ttft: token budget of a prefill round")
    side.add_argument("--vocab", type=int, default=152064,
                      help="--ttft: rows of the vocabulary matrix of the first-token head (inside the measured time); 0 stops the "
                           "clock when the prefill is complete")
    side.add_argument("--repeats", type=int, default=5, help="--ttft: timed repetitions per batch size")
    side.add_argument("--batch-sizes", type=int, nargs="*", default=[256, 512, 1024, 2048, 4096, 1 << 30], help="--ttft: values of C")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from paper_2509_24381_amd import runner
    from paper_2509_24381_amd.binding import STEPS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.short_chunks:
        return short_chunks(args)
    if args.ttft:
        return ttft_study(args)
    wl = synth.workload(args.workload)
    sh = wl.shape
    weights = [wl.weights(l) for l in range(wl.n_layers)]
    w0 = weights[0]
    if args.workload == 4:
        # one rs_prefill_batch call per step: 16 requests with imported prior caches, ragged chunks summing to the budget
        reqs = wl.batch()
        x = __import__("numpy").concatenate([r.rows for r in reqs], axis=0)
        lens = [r.rows.shape[0] for r in reqs]
        priors = [r.prior_len for r in reqs]
        visible = sum(r.prior_len + r.rows.shape[0] for r in reqs) if args.fp8_kv else 0
        stack = runner.LayerStack(sh, weights, max_tokens=wl.budget, max_requests=len(reqs), max_pos=wl.max_prior + wl.budget,
                                  fp8_visible_tokens=visible)
        kvs = []
        pool = stack.new_pool(sum((r.prior_len + r.rows.shape[0] + 63) // 64 for r in reqs), fp8=args.fp8_kv) if args.paged else None
        for r in reqs:
            kv = (pool.new_cache(1, 0.125, 0.125) if args.paged else
                  stack.new_cache_fp8(wl.max_prior + wl.budget, 0.125, 0.125) if args.fp8_kv else
                  stack.new_cache(wl.max_prior + wl.budget))
            if r.prior_len:
                kv.import_(0, runner.to_device_bf16(r.prior_k), runner.to_device_bf16(r.prior_v))
            kvs.append(kv)
        x_dev = runner.to_device_bf16(x)
        y_dev = torch.empty_like(x_dev)
        call_shapes = [(t, p) for t, p in zip(lens, priors)]          # (T_i, P_i) of the one call
        n_tokens, calls_per_step = wl.budget, 1

        def step():
            for kv, p in zip(kvs, priors):
                kv.truncate(0, p)
            stack.prefill_batch(0, kvs, lens, x_dev, y_dev)
    else:
        x = wl.prompt()
        chunks = wl.chunks()
        stack = runner.LayerStack(sh, weights, max_tokens=wl.budget, max_requests=1, max_pos=wl.n_tokens,
                                  fp8_visible_tokens=wl.n_tokens if args.fp8_kv else 0)
        pool = stack.new_pool(wl.n_layers * ((wl.n_tokens + 63) // 64), fp8=args.fp8_kv) if args.paged else None
        kv = (pool.new_cache(wl.n_layers, 0.125, 0.125) if args.paged else
              stack.new_cache_fp8(wl.n_tokens, 0.125, 0.125) if args.fp8_kv else stack.new_cache(wl.n_tokens))
        x_dev = runner.to_device_bf16(x)
        call_shapes = [(b - a, a) for a, b in chunks]
        n_tokens, calls_per_step = wl.n_tokens, len(chunks) * wl.n_layers

        def step():
            kv.reset()
            stack.prefill_prompt(x_dev, chunks, kv)
    del weights

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # every third gate/up launch is bracketed by events (all of them when a step is a single call): the samples walk
    # through all layers and chunk positions, and two thirds of the launches keep their neighbours close
    gu_every = 3 if calls_per_step > 1 else 1
    stack.ctx.profile_enable("gate_up_gemm", calls_per_step * args.steps, every=gu_every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gu_ms, gu_n = stack.ctx.profile_read()
    stack.ctx.profile_enable(None)

    layer_tokens = n_tokens * wl.n_layers
    attn_flops_step = wl.n_layers * sum(sh.attn_flops(t, p) for t, p in call_shapes)
    flops_step = wl.n_layers * sh.linear_flops_per_token() * n_tokens + attn_flops_step
    # bytes of cached K and V that attention must read per step (prefix + the chunk itself), bf16
    kv_bytes_step = wl.n_layers * sum((p + t) * 2 * sh.n_kv_heads * sh.head_dim * 2 for t, p in call_shapes)
    ms_per_step = dt / args.steps * 1e3
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12

    gu_rows = wl.budget if args.workload == 4 else max(t for t, _ in call_shapes)
    gu_rows_avg = n_tokens * wl.n_layers / calls_per_step          # rows per launch, averaged (the last chunk may be short)
    gu_flops = 2.0 * gu_rows_avg * sh.hidden * 2 * sh.mlp_inter    # per launch: [T, H] x [2I, H]^T
    gu_avg_ms = gu_ms / max(gu_n, 1)
    gu_tflops = gu_flops / (gu_avg_ms * 1e-3) / 1e12
    out = {
        "metric": "chunked-prefill tokens/s per layer @7B shape, 2048 budget; MFMA util % of peak",
        "value": layer_tokens / (ms_per_step * 1e-3),
        "unit": "layer-tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.n_layers, "tokens_per_step": n_tokens, "token_budget": wl.budget,
                   "calls_per_step": calls_per_step, "kv_cache": ("8-bit E4M3, " if args.fp8_kv else "") + ("paged (64-token pages)" if args.paged else "contiguous"),
                   "shape": f"hidden {sh.hidden}, {sh.n_q_heads} q / {sh.n_kv_heads} kv heads, head_dim {sh.head_dim}, "
                            f"mlp {sh.mlp_inter}"},
        "tflops": tflops,
        "mfma_frac_whole_path": tflops / MFMA_BF16_PEAK_TFLOPS,
        "roofline": {"kernel": f"gemm_strip_kernel<EPI_SWIGLU> (gate/up + SwiGLU, M={gu_rows} K={sh.hidden} N={2 * sh.mlp_inter})",
                     "bound": "mfma", "achieved": gu_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gu_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": GATE_UP_TRAFFIC_BYTES if args.workload == 3 else None,
                     "traffic_unit": "bytes per launch (L2/fabric boundary, rocprofv3 --pmc)",
                     "algorithmic_bytes": 2.0 * (2 * sh.mlp_inter * sh.hidden + gu_rows_avg * (sh.hidden + sh.mlp_inter)),
                     "avg_ms": gu_avg_ms, "launches": gu_n},
    }

    # one more pass per measured step of the layer, outside the timed region, every launch of that step bracketed by HIP
    # events on its stream: the attention step always (its TFLOP/s and the rate at which it reads the cached K and V),
    # every step with --breakdown
    bd = {}
    for name in (STEPS if args.breakdown else ("attention",)):
        stack.ctx.profile_enable(name, calls_per_step)
        step()
        torch.cuda.synchronize()
        ms, n = stack.ctx.profile_read()
        bd[name] = ms / max(n, 1)
    stack.ctx.profile_enable(None)
    if args.breakdown:
        out["breakdown_avg_ms_per_call"] = bd
    attn_s = bd["attention"] * 1e-3 * calls_per_step
    out["attention"] = {"kernel": "append_kv_kernel is not included; attn_prefill_pipelined_kernel (+ attn_merge_kernel when key ranges are split)",
                        "avg_ms": bd["attention"], "tflops": attn_flops_step / attn_s / 1e12,
                        "frac_of_mfma_peak": attn_flops_step / attn_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                        "kv_read_GBps": kv_bytes_step / attn_s / 1e9, "kv_read_frac_of_hbm_peak": kv_bytes_step / attn_s / 1e9 / HBM_PEAK_GBS}

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, w0, x, args.cpu_seconds)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
