#!/usr/bin/env python3
"""Benchmark of the chunked-prefill decoder-layer path on one MI355X.

A step is one pass of the whole hot path over the benchmark workload: a synthetic 8192-token multi-image prompt
(6 images of 1024 embedding rows interleaved with text spans) prefilled in 4 chunks under a 2048-token budget through
4 stacked 7B-shaped decoder layers, i.e. 16 rs_prefill_chunk calls with the KV prefix growing 0 -> 6144.
`value` = layer-tokens per second (tokens x layers / time), inputs and weights resident in HBM.
`--workload 1..5` times one of the other parity workloads the same way (4 = the 16-request ragged micro-batch through
rs_prefill_batch, 5 = the 72B-shaped layer over a 32768-token prompt); the default, 3, is the headline configuration.

Prints ONE JSON line (see README / DESIGN for the fields): metric, value, ms_per_step, roofline of the dominant
kernel (the fused gate/up + SwiGLU GEMM, timed live with HIP events on its own stream inside the timed region), and
the fp64 CPU oracle timed on a bounded sample of the same workload.
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
# Bytes crossing the L2 / fabric boundary per gate/up GEMM launch at T=2048 on the 7B shape, from the two rocprofv3 --pmc
# passes summarised in profiles/gate_up_gemm_7b_T2048_hbm_traffic_pmc.md (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the
# factors a plain copy kernel of known size gives).  Algorithmic bytes of the same launch: 363.9e6.
GATE_UP_TRAFFIC_BYTES = (466051.5 * 2.0 + 151296.0 * 1.0) * 1024


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

    if args.breakdown:
        bd = {}
        for name in STEPS:
            stack.ctx.profile_enable(name, calls_per_step)
            step()
            torch.cuda.synchronize()
            ms, n = stack.ctx.profile_read()
            bd[name] = ms / max(n, 1)
        stack.ctx.profile_enable(None)
        out["breakdown_avg_ms_per_call"] = bd
        attn_s = bd["attention"] * 1e-3 * calls_per_step
        out["attention"] = {"avg_ms": bd["attention"], "tflops": attn_flops_step / attn_s / 1e12,
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
