#!/usr/bin/env python3
"""Benchmark of the D^3 decode hot path on one MI355X.

Workload (the second benchmark configuration): Llama-7B-shaped decoder, random-init bf16
weights N(0, 0.02), batch 1, prompt of 512 uniform-random token ids, 256 greedy tokens
generated, alpha in {0.995, 1.0, 0.99}, start block 19.

One bench "step" is one request's whole generation phase: G-1 = 255 decode steps under the
D^3 schedule (every kept block, the missing-state fill of the dropped ones, lm_head, argmax),
tokens fed back on the device, no host synchronisation inside.  The prompt pass runs once,
untimed; each step rewinds the cache to the prompt with d3_truncate.  `value` is decode
tokens/s at alpha = 0.995; full depth (alpha = 1) and alpha = 0.99 are reported beside it,
each with its algorithmic HBM bytes per token and fraction of the 8 TB/s peak.

python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 7b|13b|7b-b32|70b|tiny|7b-long] [--fill copy|recompute|none]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import d3_inputs  # noqa: E402

HBM_PEAK_GBPS = 8000.0
FILL_MODES = {}

CONFIGS = {
    # name: (shape, B, P, G, alphas (first is the headline), start fraction)
    "tiny": (d3_inputs.TINY, 1, 16, 32, (0.97, 1.0), 0.6),
    "7b": (d3_inputs.LLAMA_7B, 1, 512, 256, (0.995, 1.0, 0.99), 0.6),
    "13b": (d3_inputs.LLAMA_13B, 4, 1024, 256, (0.995, 1.0), 0.6),
    "7b-b32": (d3_inputs.LLAMA_7B, 32, 2048, 512, (0.995, 1.0), 0.6),
    "70b": (d3_inputs.LLAMA_70B, 8, 1024, 256, (0.995, 1.0), 0.6),
    # a long-generation shape beside the benchmark's five: the paper's GSM8K setting (maximum length 1024,
    # alpha = 0.9999, start = 0.2, batch 4 for the 7B model; Section 4.1 and 4.2)
    "7b-long": (d3_inputs.LLAMA_7B, 4, 512, 1024, (0.9999, 1.0), 0.2),
    # a batch of unequal few-shot prompts, padded on the left to the longest as an evaluation harness batches them
    # (Section 4.2); every sequence attends to its own rows only
    "7b-ragged": (d3_inputs.LLAMA_7B, 4, 512, 256, (0.995, 1.0), 0.6),
}
RAGGED_LENGTHS = {"7b-ragged": (512, 384, 256, 128)}


def block_weight_bytes(s) -> int:
    return s.params_per_block * (4 if s.dtype == "f32" else 2)


def algorithmic_bytes(s, B, P, G, keep, kv_bytes_per_elem, fill="copy", prompt_rows=None):
    """HBM bytes the method must move over decode steps 1..G-1: weights of the executed blocks,
    their KV rows read and appended, the fill of the dropped blocks (COPY: read one row, write it;
    RECOMPUTE: stream W_k and W_v of every dropped block, write its row), lm_head.
    prompt_rows: prompt rows of the whole batch when the prompts are unequal (default B * P)."""
    wb = block_weight_bytes(s)
    kv_row = 2 * s.H_kv * s.hd * kv_bytes_per_elem          # K + V of one token in one block
    head = s.V * s.d * (4 if s.dtype == "f32" else 2)
    total = 0
    for i in range(1, G):
        k, n = int(keep[i]), s.L - int(keep[i])
        per_dropped = {"copy": 2 * kv_row * B, "none": 0,
                       "recompute": 2 * s.H_kv * s.hd * s.d * (4 if s.dtype == "f32" else 2) + kv_row * B}[fill]
        rows = (B * P if prompt_rows is None else prompt_rows) + B * i
        total += k * (wb + kv_row * rows + kv_row * B) + n * per_dropped + head
    return total


def run_decode(dec, torch, first_tok, P, G, alpha, start, requests, fill="copy", table=None):
    """`requests` whole generation phases back to back; returns seconds (host clock around a device sync).
    table: (keep, drop_begin) of a schedule to follow instead of the power law."""
    cur = first_tok.clone()
    nxt = torch.zeros_like(cur)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(requests):
        dec.truncate(P)
        if table is not None:
            dec.set_plan_table(table[0], table[1])
        else:
            dec.set_plan(alpha, start, 0, G)
        cur.copy_(first_tok)
        for i in range(1, G):
            dec.decode_step(cur, i, nxt)
            if fill != "none":
                dec.fill_missing_kv(P + i - 1, P + i, FILL_MODES[fill])
            cur, nxt = nxt, cur
    dec.synchronize()
    return time.perf_counter() - t0


def cpu_baseline(shape, keep_mean):
    """The oracle (float32 build, one thread) on a one-block model of the same widths; per-block and
    lm_head times extrapolated to the workload's average depth."""
    from oracle import oracle
    s1 = shape.truncated(1)
    w = d3_inputs.make_weights(s1, 0)
    model = oracle.OracleModel(s1, w, "f32")
    oracle.set_threads(1, "f32")
    cap = 256                                   # a bounded sample: about 9 s of block steps and 3 s of lm_head passes
    seq = model.new_seq(2 * cap)
    toks = d3_inputs.make_prompt(1, 2 * cap, s1.V, seed=3)[0]
    n_block, t0 = 0, time.perf_counter()
    while n_block < cap and (n_block < 4 or time.perf_counter() - t0 < 9.0):
        seq.forward_token(int(toks[n_block]), n_block, [0])
        n_block += 1
    t_block = (time.perf_counter() - t0) / n_block
    n_head, t0 = 0, time.perf_counter()
    while n_head < cap and (n_head < 2 or time.perf_counter() - t0 < 3.0):
        seq.forward_token(int(toks[n_block + n_head]), n_block + n_head, [], want_logits=True)
        n_head += 1
    t_head = (time.perf_counter() - t0) / n_head
    per_tok = keep_mean * t_block + t_head
    return {"value": 1.0 / per_tok, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"float32 oracle, 1 thread, {s1.name}: {n_block} block-steps ({t_block * 1e3:.0f} ms each) + {n_head} lm_head "
                      f"passes ({t_head * 1e3:.0f} ms each), extrapolated to {keep_mean:.2f} blocks/token",
            "host_cores_available": os.cpu_count()}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="7b", choices=sorted(CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fill", action="store_true", help="same as --fill none")
    ap.add_argument("--fill", default="copy", choices=["copy", "recompute", "none"],
                    help="missing-state fill after every decode step (Section 3.2): KV copy (default), KV recompute, or none")
    ap.add_argument("--compare-schedules", action="store_true",
                    help="also time the comparison schedules of Section 4.1 at the headline alpha's average depth: the same "
                         "power law with deep blocks dropped first, and linear decay with shallow blocks dropped first")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2503_08524_amd import binding
    FILL_MODES.update(copy=binding.D3_FILL_COPY, recompute=binding.D3_FILL_RECOMPUTE)
    fill = "none" if args.no_fill else args.fill

    shape, B, P, G, alphas, start_frac = CONFIGS[args.config]
    start = d3_inputs.start_layer_from_fraction(shape.L, start_frac)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    kv = "f32" if shape.dtype == "f32" else "f16"
    weights = binding.random_weights_on_device(shape, 0, dev)
    dec = binding.Decoder(shape, weights, B, P + G, kv_dtype=kv, device=dev)
    prompts = torch.from_numpy(d3_inputs.make_prompt(B, P, shape.V, seed=1)).to(dev)

    # a plain device-to-device copy of known size (1 GiB read + 1 GiB written): the yardstick that scales the
    # FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    # the same copy, timed: what a plain streaming kernel reaches on this chip (bytes read + bytes written per second),
    # the ceiling that the fractions of the nominal 8 TB/s can be held against
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(5):
        cal_dst.copy_(cal_src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * (1 << 30) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del cal_src, cal_dst

    dec.set_plan(alphas[0], start, 0, G)
    if fill == "recompute":
        dec.set_fill_mode(binding.D3_FILL_RECOMPUTE)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    lengths = RAGGED_LENGTHS.get(args.config)
    first_tok = dec.prefill_ragged(prompts, lengths) if lengths else dec.prefill(prompts)
    prompt_rows = sum(lengths) if lengths else None
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0

    kv_bytes = 4 if kv == "f32" else 2
    results = {}
    for alpha in alphas:
        keep, _, _ = binding.d3_plan_depth(shape.L, alpha, start, 0, G)
        run_decode(dec, torch, first_tok, P, G, alpha, start, args.warmup, fill)
        secs = run_decode(dec, torch, first_tok, P, G, alpha, start, args.steps, fill)
        n_tok = args.steps * (G - 1) * B
        alg = algorithmic_bytes(shape, B, P, G, keep, kv_bytes, fill, prompt_rows) * args.steps
        results[alpha] = {
            "tokens_per_s": n_tok / secs, "ms_per_token_step": secs / (args.steps * (G - 1)) * 1e3,
            "avg_blocks": float(keep[1:G].mean()), "algorithmic_GB_per_token_step": alg / (args.steps * (G - 1)) / 1e9,
            "achieved_GBps": alg / secs / 1e9, "frac_of_hbm_peak": alg / secs / 1e9 / HBM_PEAK_GBPS,
            "frac_of_measured_copy_rate": alg / secs / 1e9 / copy_gbps,
        }
    head = results[alphas[0]]
    if 1.0 in results:
        for a, r in results.items():
            r["speedup_vs_full_depth"] = r["tokens_per_s"] / results[1.0]["tokens_per_s"]
            r["ideal_layer_count_ratio"] = shape.L / r["avg_blocks"]
            r["ideal_byte_ratio"] = results[1.0]["algorithmic_GB_per_token_step"] / r["algorithmic_GB_per_token_step"]

    schedules = None
    if args.compare_schedules and 1.0 in results:
        # Same kernels, other plans (Section 4.1's comparison methods as far as the paper defines them: which blocks go
        # first, and linear instead of power-law decay between bounds chosen to give at least the same average depth).
        L = shape.L
        d3_keep, d3_drop, _ = binding.d3_plan_depth(L, alphas[0], start, 0, G)
        avg = float(d3_keep[1:G].mean())
        last = max(0, min(L, int(2 * avg - L)))
        while last < L and float(binding.d3_plan_depth_linear(L, L, last, 0, G)[0][1:G].mean()) < avg:
            last += 1
        plans = {"power law, middle blocks first (D^3)": (d3_keep, d3_drop),
                 "power law, deep blocks first (early exit)": binding.d3_plan_depth(L, alphas[0], L - 1, 0, G)[:2],
                 "linear %d -> %d, shallow blocks first" % (L, last): binding.d3_plan_depth_linear(L, L, last, 0, G)[:2]}
        schedules = {}
        for name, table in plans.items():
            run_decode(dec, torch, first_tok, P, G, 1.0, start, args.warmup, fill, table=table)
            secs = run_decode(dec, torch, first_tok, P, G, 1.0, start, args.steps, fill, table=table)
            k = table[0]
            schedules[name] = {"avg_blocks": float(k[1:G].mean()), "tokens_per_s": args.steps * (G - 1) * B / secs,
                               "speedup_vs_full_depth": args.steps * (G - 1) * B / secs / results[1.0]["tokens_per_s"],
                               "ideal_layer_count_ratio": L / float(k[1:G].mean())}

    # dominant kernel, every launch bracketed by HIP events on the launch stream, over one more full-depth request
    wbytes = 4 if shape.dtype == "f32" else 2
    if args.config == "7b-b32":
        # at batch 32 the cache rows outweigh the weights: attention is the dominant kernel (one launch per block;
        # bytes averaged over the request's steps: K and V rows of B sequences, read once)
        kernel = "decode attention (RoPE + KV append + split merge included)"
        kv_row = 2 * shape.H_kv * shape.hd * kv_bytes
        kclass, bytes_per_launch = binding.D3_K_ATTN, sum(B * (P + i) * kv_row for i in range(1, G)) / (G - 1) + 2 * B * shape.d * 4
    else:
        kernel = "fused RMSNorm + gate/up + SiLU*mul projection"
        kclass, bytes_per_launch = binding.D3_K_GATE_UP, 2 * shape.F * shape.d * wbytes + B * shape.d * 4 + B * shape.F * 4
    dec.profile_select(kclass)
    run_decode(dec, torch, first_tok, P, G, 1.0, start, 1, "none")
    ms, n = dec.profile_read()
    dec.profile_select(binding.D3_K_NONE)
    achieved = bytes_per_launch / (ms / n * 1e-3) / 1e9 if n else 0.0
    # HBM bytes per launch of that kernel from the committed rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE,
    # each scaled by what a plain 1 GiB copy reads on the same counter); only known for the profiled workload
    traffic = None
    profiled = {"7b": ("decode_7b_b1", "gemv_alu_kernel<unsigned short, 1, 2, true>"),       # gate/up kernel of each configuration
                "13b": ("decode_13b_b4", "gemm_mfma_kernel<1, 2, 2, true>"),
                "70b": ("decode_70b_b8", "gemm_mfma_kernel<1, 2, 1, true>")}
    if args.config in profiled and kclass == binding.D3_K_GATE_UP:
        stem, kname = profiled[args.config]
        tpath = os.path.join(ROOT, "profiles", stem + "_hbm_traffic.json")
        if os.path.exists(tpath):
            with open(tpath) as f:
                ks = [v for name, v in json.load(f)["kernels"].items() if kname in name]
            if ks and ks[0]["write_bytes_per_launch"] is not None:
                traffic = ks[0]["fetch_bytes_per_launch"] + ks[0]["write_bytes_per_launch"]
    roofline = {"bound": "hbm", "kernel": kernel, "achieved": achieved,
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                "launches_timed": n, "avg_launch_us": ms / n * 1e3 if n else None, "bytes_per_launch": bytes_per_launch}

    out = {
        "metric": "decode tokens/sec (D^3, alpha=%g) at the Llama-7B shape; achieved HBM GB/s beside it" % alphas[0]
        if args.config == "7b" else "decode tokens/sec (D^3, alpha=%g)" % alphas[0],
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_token_step"] * (G - 1), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if shape.dtype == "f32" else "bf16 weights, f32 accumulate, f16 KV cache",
        "data": "synthetic",
        "config": {"workload": f"{shape.name} B={B} P={P if not lengths else list(lengths)} G={G} alpha={alphas[0]} start_layer={start}",
                   "step": f"one request's generation phase = {G - 1} decode steps", "kv_cache": kv,
                   "fill_every_step": fill},
        "ms_per_token": head["ms_per_token_step"], "prefill_s": prefill_s,
        "by_alpha": {str(a): r for a, r in results.items()},
        "stream_copy": {"GBps": copy_gbps, "what": "1 GiB device-to-device copy, read + written bytes per second (5 repeats)"},
        "roofline": roofline,
    }
    if schedules is not None:
        out["schedules"] = schedules
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, head["avg_blocks"])
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
