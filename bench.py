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

Beside the headline the line carries: `kernels` (every kernel class of a block at full depth: microseconds per launch
between HIP events on the launch stream, algorithmic bytes, fraction of the 8 TB/s peak), `roofline` (the dominant
kernel, same clock), a read-only streaming yardstick (`stream_read`), the prompt pass against the bf16 matrix-core
peak and against what the matrix cores sustain on this chip (`prefill`, `prefill.sustained_TFLOPs`), and `by_config`: the 13B (batch 4), 7B batch-32 and 70B (batch 8) configurations, each with full
depth and D^3, two timed requests each (skip them with --no-extra-configs).

python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 7b|13b|7b-b32|70b|tiny|7b-long|7b-ragged]
                [--fill copy|recompute|none] [--no-extra-configs] [--no-cpu-baseline] [--kv f16|f32]
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
MFMA_BF16_PEAK_TFLOPS = 2500.0
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


def kernel_bytes(s, B, P, G, kv_bytes_per_elem):
    """Algorithmic bytes one launch of each kernel class moves at batch B (weights once, activations in and out;
    attention: the K and V rows of B sequences averaged over the request's steps, q in, output out)."""
    wb = 4 if s.dtype == "f32" else 2
    qdim, kvdim = s.H * s.hd, s.H_kv * s.hd
    kv_row = 2 * kvdim * kv_bytes_per_elem
    return {
        "qkv": (qdim + 2 * kvdim) * s.d * wb + B * s.d * 4 + B * (qdim + 2 * kvdim) * 4,
        "attn": sum(B * (P + i) * kv_row for i in range(1, G)) / (G - 1) + 2 * B * qdim * 4,
        "o": s.d * qdim * wb + B * qdim * 4 + 2 * B * s.d * 4,
        "gate_up": 2 * s.F * s.d * wb + B * s.d * 4 + B * s.F * 4,
        "down": s.d * s.F * wb + B * s.F * 4 + 2 * B * s.d * 4,
        "lm_head": s.V * s.d * wb + B * s.d * 4 + B * s.V * 4,
    }


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
            dec.set_plan(alpha, start, 0, G)          # host only: the schedule of the request
        cur.copy_(first_tok)
        for i in range(1, G):
            dec.decode_step(cur, i, nxt)
            if fill != "none":
                dec.fill_missing_kv(P + i - 1, P + i, FILL_MODES[fill])
            cur, nxt = nxt, cur
    dec.synchronize()
    return time.perf_counter() - t0


def yardsticks(dec, torch, dev):
    """A plain 1 GiB device-to-device copy (read + written bytes per second; it also scales the FETCH_SIZE / WRITE_SIZE
    counters when this command runs under rocprofv3 --pmc) and a read-only stream over 2 GiB with the projections' own
    load instructions and launch shape: what the memory system gives a kernel that only reads."""
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(5):
        cal_dst.copy_(cal_src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * (1 << 30) / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del cal_dst
    big = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    big.zero_()
    out = {}
    # sizes of the 7B shape's matrices beside the large ones: O-projection 32 MiB, down-projection 86 MiB, QKV 96 MiB,
    # gate/up 172 MiB, lm_head 250 MiB (a launch's fixed costs weigh more the smaller its matrix)
    sizes = (("2 GiB", 2 << 30), ("1 GiB", 1 << 30), ("250 MiB", 250 << 20), ("172 MiB", 172 << 20), ("96 MiB", 96 << 20),
             ("86 MiB", 86 << 20), ("32 MiB", 32 << 20))
    for name, nbytes in sizes:
        t = big[:nbytes]
        dec.stream_read(t)
        torch.cuda.synchronize()
        # each launch reads a different window of the 2 GiB buffer (as every projection of a step reads different weights:
        # nothing comes from a cache), launches back to back on the stream
        n = 5 if nbytes >= (1 << 30) else 40
        windows = [big[(i * nbytes) % ((2 << 30) - nbytes + 1) // 256 * 256:][:nbytes] for i in range(n)]
        ev0.record()
        for w in windows:
            dec.stream_read(w)
        ev1.record()
        torch.cuda.synchronize()
        out[name] = n * nbytes / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del big, cal_src
    return copy_gbps, out


def progress(msg):
    """Progress lines go to stderr (stdout carries the one JSON line); a long run must not stay silent."""
    print("bench: " + msg, file=sys.stderr, flush=True)


def measure_config(name, steps, warmup, fill, kv_arg=None, with_yardsticks=False, compare_schedules=False):
    """Everything measured for one configuration; frees its device memory before returning."""
    import torch
    from paper_2503_08524_amd import binding
    shape, B, P, G, alphas, start_frac = CONFIGS[name]
    start = d3_inputs.start_layer_from_fraction(shape.L, start_frac)
    dev = "cuda:0"
    kv = kv_arg or binding.default_kv_dtype(shape)
    progress(f"{name}: drawing weights on the device")
    weights = binding.random_weights_on_device(shape, 0, dev)
    dec = binding.Decoder(shape, weights, B, P + G, kv_dtype=kv, device=dev)
    prompts = torch.from_numpy(d3_inputs.make_prompt(B, P, shape.V, seed=1)).to(dev)
    res = {"kv_cache": kv}
    if with_yardsticks:
        res["stream_copy_GBps"], res["stream_read_GBps"] = yardsticks(dec, torch, dev)

    dec.set_plan(alphas[0], start, 0, G)
    if fill == "recompute":
        dec.set_fill_mode(binding.D3_FILL_RECOMPUTE)
    lengths = RAGGED_LENGTHS.get(name)
    prompt_rows = sum(lengths) if lengths else None
    prefill = (lambda: dec.prefill_ragged(prompts, lengths)) if lengths else (lambda: dec.prefill(prompts))
    progress(f"{name}: prompt pass, {prompt_rows or B * P} tokens (after one sequence alone, which pages the kernels in)")
    dec.prefill(prompts[:1, P - (lengths[0] if lengths else P):].contiguous())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    first_tok = prefill()
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    progress(f"{name}: prompt pass took {prefill_s:.3f} s")
    n_prompt = prompt_rows or B * P
    # matrix-core work of the prompt pass: 2 flops per weight per token (lm_head once per sequence) plus the causal
    # attention contractions; the kernels issue twice that (activations go in as bf16 hi + lo)
    attn_flops = sum(4 * shape.H * shape.hd * (p + 1) for p in range(P)) * B * shape.L if not lengths else 0
    flops = 2.0 * shape.params_per_block * shape.L * n_prompt + 2.0 * shape.V * shape.d * B + attn_flops
    res["prefill"] = {"tokens": n_prompt, "seconds": prefill_s, "tokens_per_s": n_prompt / prefill_s,
                      "algorithmic_TFLOPs": flops / prefill_s / 1e12, "issued_TFLOPs_hi_lo": 2 * flops / prefill_s / 1e12,
                      "bound": "mfma", "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                      "frac_algorithmic": flops / prefill_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                      "frac_issued": 2 * flops / prefill_s / 1e12 / MFMA_BF16_PEAK_TFLOPS}

    if with_yardsticks:
        # what the matrix cores sustain on this chip: the stage loop of the prompt GEMM on fixed operands (d3_mfma_yardstick)
        n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
        sustained = {}
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for mode, label in ((0, "mfma_alone"), (1, "with_lds_fragment_reads"), (2, "with_reads_and_stage_barrier")):
            dec.mfma_yardstick(mode, 1024)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(3):
                dec.mfma_yardstick(mode, 4096)
            e1.record()
            torch.cuda.synchronize()
            sustained[label] = 3 * n_cu * 8 * 4096 * 32 * 16384 / (e0.elapsed_time(e1) * 1e-3) / 1e12
        res["prefill"]["sustained_TFLOPs"] = sustained
        res["prefill"]["frac_issued_of_sustained_mfma_alone"] = res["prefill"]["issued_TFLOPs_hi_lo"] / sustained["mfma_alone"]
        progress(f"{name}: matrix cores sustain {sustained['mfma_alone']:.0f} TFLOP/s alone, {sustained['with_reads_and_stage_barrier']:.0f} in the prompt GEMM's stage loop")

    kv_bytes = 4 if kv == "f32" else 2
    results = {}
    for alpha in alphas:
        keep, _, _ = binding.d3_plan_depth(shape.L, alpha, start, 0, G)
        run_decode(dec, torch, first_tok, P, G, alpha, start, warmup, fill)
        secs = run_decode(dec, torch, first_tok, P, G, alpha, start, steps, fill)
        n_tok = steps * (G - 1) * B
        alg = algorithmic_bytes(shape, B, P, G, keep, kv_bytes, fill, prompt_rows) * steps
        progress(f"{name}: alpha {alpha}: {n_tok / secs:.1f} tokens/s, {secs / (steps * (G - 1)) * 1e3:.3f} ms per decode step")
        results[alpha] = {
            "tokens_per_s": n_tok / secs, "ms_per_token_step": secs / (steps * (G - 1)) * 1e3,
            "avg_blocks": float(keep[1:G].mean()), "algorithmic_GB_per_token_step": alg / (steps * (G - 1)) / 1e9,
            "achieved_GBps": alg / secs / 1e9, "frac_of_hbm_peak": alg / secs / 1e9 / HBM_PEAK_GBPS,
        }
    if 1.0 in results:
        for a, r in results.items():
            r["speedup_vs_full_depth"] = r["tokens_per_s"] / results[1.0]["tokens_per_s"]
            r["ideal_layer_count_ratio"] = shape.L / r["avg_blocks"]
            r["ideal_byte_ratio"] = results[1.0]["algorithmic_GB_per_token_step"] / r["algorithmic_GB_per_token_step"]
    res["by_alpha"] = {str(a): r for a, r in results.items()}

    if compare_schedules and 1.0 in results:
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
        for pname, table in plans.items():
            run_decode(dec, torch, first_tok, P, G, 1.0, start, warmup, fill, table=table)
            secs = run_decode(dec, torch, first_tok, P, G, 1.0, start, steps, fill, table=table)
            k = table[0]
            schedules[pname] = {"avg_blocks": float(k[1:G].mean()), "tokens_per_s": steps * (G - 1) * B / secs,
                                "speedup_vs_full_depth": steps * (G - 1) * B / secs / results[1.0]["tokens_per_s"],
                                "ideal_layer_count_ratio": L / float(k[1:G].mean())}
        res["schedules"] = schedules

    # every kernel class of a block, each launch bracketed by two HIP events on the launch stream, over one more
    # full-depth request per class; the empty bracket (no launch inside) is what the event pair itself adds
    kb = kernel_bytes(shape, B, P, G, kv_bytes)
    classes = {"qkv": binding.D3_K_QKV, "attn": binding.D3_K_ATTN, "o": binding.D3_K_OPROJ, "gate_up": binding.D3_K_GATE_UP,
               "down": binding.D3_K_DOWN, "lm_head": binding.D3_K_LM_HEAD, "empty_bracket": binding.D3_K_EMPTY}
    kernels = {}
    for cname, cls in classes.items():
        dec.profile_select(cls)
        run_decode(dec, torch, first_tok, P, G, 1.0, start, 1, "none")
        ms, n = dec.profile_read()
        us = ms / n * 1e3 if n else None
        kernels[cname] = {"us_per_launch": us, "launches": n}
        progress(f"{name}: kernel class {cname}: {us if us is None else round(us, 2)} us per launch")
    dec.profile_select(binding.D3_K_NONE)
    pair_us = kernels["empty_bracket"]["us_per_launch"] or 0.0
    for cname, k in kernels.items():
        if cname == "empty_bracket" or not k["launches"]:
            continue
        k["bytes_per_launch"] = kb[cname]
        k["GBps"] = kb[cname] / (k["us_per_launch"] * 1e-6) / 1e9
        k["frac_of_hbm_peak"] = k["GBps"] / HBM_PEAK_GBPS
        k["us_minus_event_pair"] = k["us_per_launch"] - pair_us
        k["frac_minus_event_pair"] = kb[cname] / (k["us_minus_event_pair"] * 1e-6) / 1e9 / HBM_PEAK_GBPS
    res["kernels"] = kernels
    res["dominant"] = "attn" if name == "7b-b32" else "gate_up"
    dec.close()
    del dec, weights, prompts, first_tok
    torch.cuda.empty_cache()
    return res


def cpu_baseline(shape, keep_mean):
    """The oracle (float32 build, one thread) on a one-block model of the same widths; per-block and
    lm_head times extrapolated to the workload's average depth."""
    from oracle import oracle
    s1 = shape.truncated(1)
    progress("cpu_baseline: drawing one block on the host")
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
    ap.add_argument("--kv", default=None, choices=["f16", "f32"], help="KV cache precision (default: by model depth)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-configs", action="store_true", help="skip the by_config entries (13b, 7b-b32, 70b)")
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
    torch.cuda.set_device(0)

    shape, B, P, G, alphas, start_frac = CONFIGS[args.config]
    start = d3_inputs.start_layer_from_fraction(shape.L, start_frac)
    lengths = RAGGED_LENGTHS.get(args.config)
    m = measure_config(args.config, args.steps, args.warmup, fill, args.kv, with_yardsticks=True,
                       compare_schedules=args.compare_schedules)
    head = m["by_alpha"][str(alphas[0])]
    dom = m["kernels"][m["dominant"]]
    kernel_names = {"gate_up": "fused RMSNorm + gate/up + SiLU*mul projection",
                    "attn": "decode attention (RoPE + KV append + split merge included)"}
    # HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc runs of this command (FETCH_SIZE +
    # WRITE_SIZE, each scaled by what a plain 1 GiB copy reads on the same counter); only known for a profiled workload
    traffic, traffic_source = None, None
    profiled = {"7b": ("decode_7b_b1", "gemv_alu_kernel<unsigned short, 1, 2, true>"),
                "13b": ("decode_13b_b4", "gemm_mfma_kernel<1, 2, 2, true>"),
                "70b": ("decode_70b_b8", "gemm_mfma_kernel<1, 2, 1, true>")}
    if args.config in profiled and m["dominant"] == "gate_up":
        stem, kname = profiled[args.config]
        tpath = os.path.join(ROOT, "profiles", stem + "_hbm_traffic.json")
        if os.path.exists(tpath):
            with open(tpath) as f:
                ks = [v for name, v in json.load(f)["kernels"].items() if kname in name]
            if ks and ks[0]["write_bytes_per_launch"] is not None:
                traffic = ks[0]["fetch_bytes_per_launch"] + ks[0]["write_bytes_per_launch"]
                traffic_source = "profiles/%s_hbm_traffic.json (committed rocprofv3 --pmc runs of this command, not this run)" % stem
    roofline = {"bound": "hbm", "kernel": kernel_names[m["dominant"]], "achieved": dom["GBps"], "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": dom["frac_of_hbm_peak"], "traffic": traffic, "traffic_source": traffic_source,
                "clock": "HIP events recorded on the launch stream around every launch of the kernel (full-depth request); "
                         "the pair of events adds kernels.empty_bracket.us_per_launch to each, which the kernel trace in profiles/ "
                         "does not see: frac_minus_event_pair is the same figure without it",
                "launches_timed": dom["launches"], "avg_launch_us": dom["us_per_launch"],
                "avg_launch_us_minus_event_pair": dom["us_minus_event_pair"], "frac_minus_event_pair": dom["frac_minus_event_pair"],
                "bytes_per_launch": dom["bytes_per_launch"]}
    copy_gbps = m["stream_copy_GBps"]
    if args.config in ("7b", "7b-long", "7b-ragged"):
        # each projection against a pure read of a buffer of its matrix's size, launched back to back the same way
        same_size = {"o": "32 MiB", "down": "86 MiB", "qkv": "96 MiB", "gate_up": "172 MiB", "lm_head": "250 MiB"}
        for cname, label in same_size.items():
            k = m["kernels"][cname]
            if k.get("launches"):
                k["pure_read_of_its_size_GBps"] = m["stream_read_GBps"][label]
                k["frac_of_pure_read_of_its_size"] = k["GBps"] / m["stream_read_GBps"][label]
    for r in m["by_alpha"].values():
        r["frac_of_measured_read_rate"] = r["achieved_GBps"] / m["stream_read_GBps"]["2 GiB"]

    out = {
        "metric": "decode tokens/sec (D^3, alpha=%g) at the Llama-7B shape; achieved HBM GB/s beside it" % alphas[0]
        if args.config == "7b" else "decode tokens/sec (D^3, alpha=%g)" % alphas[0],
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_token_step"] * (G - 1), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if shape.dtype == "f32" else "bf16 weights, f32 accumulate, %s KV cache" % m["kv_cache"],
        "data": "synthetic",
        "config": {"workload": f"{shape.name} B={B} P={P if not lengths else list(lengths)} G={G} alpha={alphas[0]} start_layer={start}",
                   "step": f"one request's generation phase = {G - 1} decode steps", "kv_cache": m["kv_cache"],
                   "fill_every_step": fill},
        "ms_per_token": head["ms_per_token_step"], "prefill_s": m["prefill"]["seconds"], "prefill": m["prefill"],
        "by_alpha": m["by_alpha"],
        "stream_copy": {"GBps": copy_gbps, "what": "1 GiB device-to-device copy, read + written bytes per second (5 repeats)"},
        "stream_read": {"GBps": m["stream_read_GBps"],
                        "what": "read-only stream with the projections' load instructions and launch shape (d3_stream_read), "
                                "bytes read per second by buffer size"},
        "roofline": roofline,
        "kernels": m["kernels"],
    }
    if "schedules" in m:
        out["schedules"] = m["schedules"]
    if not args.no_extra_configs and args.config == "7b":
        # the other benchmark configurations, two timed requests each after one warm-up request
        by_config = {}
        for name in ("13b", "7b-b32", "70b"):
            e = measure_config(name, 2, 1, fill)
            s2, B2, P2, G2, al2, _ = CONFIGS[name]
            d2 = e["kernels"][e["dominant"]]
            by_config[name] = {"workload": f"{s2.name} B={B2} P={P2} G={G2}", "kv_cache": e["kv_cache"], "timed_requests": 2,
                               "by_alpha": e["by_alpha"], "prefill": e["prefill"],
                               "dominant_kernel": {"class": e["dominant"], "us_per_launch": d2["us_per_launch"],
                                                   "bytes_per_launch": d2["bytes_per_launch"], "frac_of_hbm_peak": d2["frac_of_hbm_peak"],
                                                   "frac_minus_event_pair": d2["frac_minus_event_pair"]},
                               "kernels": {k: {kk: v.get(kk) for kk in ("us_per_launch", "frac_of_hbm_peak")} for k, v in e["kernels"].items()}}
        out["by_config"] = by_config
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, head["avg_blocks"])
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
