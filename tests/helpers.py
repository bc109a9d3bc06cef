"""Shared by the GPU parity tests: run the HIP path and the oracle on the same seeded inputs."""
from __future__ import annotations

import os
from typing import Optional

import numpy as np

import d3_inputs
from oracle import oracle

LOGIT_ATOL = 2e-2        # max abs error of logits, bf16 GPU path vs oracle (the stated acceptance bound)
HIDDEN_REL_L2 = 1e-2     # relative L2 error of the hidden state after every executed block
TOKEN_MARGIN = 10 * LOGIT_ATOL   # tokens must agree wherever the oracle's top-2 gap exceeds this


def oracle_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def gpu_generate(shape, w_np, prompts: np.ndarray, G: int, alpha: float, start: int, forced: Optional[np.ndarray] = None,
                 kv_dtype: Optional[str] = None, max_seq: Optional[int] = None, min_keep: int = 0, fill_each_step: bool = False,
                 decoder=None, pos_begin: int = 0, max_batch: Optional[int] = None,
                 fill_mode: int = 0, linear=None, lengths=None):
    """Prompt pass + G-1 decode steps through the C ABI.  forced: [B][G-1] tokens fed instead of the GPU's own.
    linear: (keep_first, keep_last) of a linear-decay schedule to follow instead of the power law.
    lengths: [B] prompt lengths of a left-padded batch (prompts[b, P - lengths[b]:] are sequence b's tokens).
    Returns dict(tokens [G][B], logits [G][B][V], hidden: list of [(k_i+1)][B][d], decoder)."""
    import torch
    from paper_2503_08524_amd import binding

    B, P = prompts.shape
    dev = "cuda:0"
    if decoder is None:
        w_dev = binding.weights_to_device(shape, w_np, dev)
        decoder = binding.Decoder(shape, w_dev, max_batch or B, max_seq or (pos_begin + P + G), kv_dtype=kv_dtype, device=dev)
    L = shape.L
    if linear is not None:
        keep, drop, _ = binding.d3_plan_depth_linear(L, linear[0], linear[1], start, max(G, 2))
        decoder.set_plan_table(keep, drop)
    else:
        keep, _, _ = binding.d3_plan_depth(L, alpha, start, min_keep, max(G, 2))
        decoder.set_plan(alpha, start, min_keep, max(G, 2))
    decoder.set_fill_mode(fill_mode)
    toks = torch.from_numpy(np.ascontiguousarray(prompts, np.int32)).to(dev)
    logits = torch.zeros(B, shape.V, dtype=torch.float32, device=dev)
    hid = torch.zeros(L + 1, B, shape.d, dtype=torch.float32, device=dev)
    if lengths is not None:
        cur = decoder.prefill_ragged(toks, lengths, logits=logits, hidden_dump=hid)
    else:
        cur = decoder.prefill(toks, pos_begin=pos_begin, logits=logits, hidden_dump=hid)
    out_tokens = [cur.cpu().numpy().copy()]
    out_logits = [logits.cpu().numpy().copy()]
    out_hidden = [hid.cpu().numpy().copy()]
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    for i in range(1, G):
        if forced is not None:
            cur = torch.from_numpy(np.ascontiguousarray(forced[:, i - 1], np.int32)).to(dev)
        k = int(keep[i])
        hid_i = torch.zeros(k + 1, B, shape.d, dtype=torch.float32, device=dev)
        decoder.decode_step(cur, i, nxt, logits=logits, hidden_dump=hid_i)
        if fill_each_step:
            decoder.fill_missing_kv(decoder.n_ctx - 1, decoder.n_ctx, fill_mode)
        cur = nxt.clone()
        out_tokens.append(cur.cpu().numpy().copy())
        out_logits.append(logits.cpu().numpy().copy())
        out_hidden.append(hid_i.cpu().numpy().copy())
    decoder.synchronize()
    return {"tokens": np.stack(out_tokens), "logits": np.stack(out_logits), "hidden": out_hidden, "decoder": decoder}


def oracle_generate(shape, w_np, prompts: np.ndarray, G: int, alpha: float, start: int, forced=None, min_keep: int = 0,
                    max_seq: Optional[int] = None, variant: str = "f64", linear=None, lengths=None):
    """One oracle Generation per sequence (sequences of a batch are independent and share the schedule)."""
    oracle.set_threads(oracle_threads(), variant)
    model = oracle.OracleModel(shape, w_np, variant)
    gens = []
    plan = None if linear is None else oracle.plan_depth_linear(shape.L, linear[0], linear[1], start, max(G, 2), variant)
    for b in range(prompts.shape[0]):
        own = prompts[b] if lengths is None else prompts[b, prompts.shape[1] - int(lengths[b]):]   # a sequence knows nothing of its padding
        gens.append(oracle.generate(model, own, G, alpha, start, min_keep=min_keep, max_seq=max_seq,
                                    forced=None if forced is None else forced[b], plan=plan))
    return model, gens


def compare(gpu, gens, G: int, check_tokens: str = "margin", logit_atol: float = LOGIT_ATOL, hidden_tol: float = HIDDEN_REL_L2):
    """Element-by-element comparison.  check_tokens: 'all' (must be identical), 'margin' (identical wherever the
    oracle's top-2 gap exceeds TOKEN_MARGIN), 'none'."""
    worst_logit, worst_hidden = 0.0, 0.0
    for b, gen in enumerate(gens):
        for i in range(G):
            ref = gen.logits[i]
            got = gpu["logits"][i][b].astype(np.float64)
            err = float(np.abs(got - ref).max())
            worst_logit = max(worst_logit, err)
            assert err <= logit_atol, f"logits seq {b} step {i}: max abs err {err:.3e}"
            hr, hg = gen.hidden[i], gpu["hidden"][i][:, b, :].astype(np.float64)
            assert hr.shape == hg.shape, (hr.shape, hg.shape)
            for e in range(hr.shape[0]):
                rel = float(np.linalg.norm(hg[e] - hr[e]) / np.linalg.norm(hr[e]))
                worst_hidden = max(worst_hidden, rel)
                assert rel <= hidden_tol, f"hidden seq {b} step {i} slot {e}: rel L2 {rel:.3e}"
            top2 = np.partition(ref, -2)[-2:]
            margin = float(top2[1] - top2[0])
            if check_tokens == "all" or (check_tokens == "margin" and margin > TOKEN_MARGIN):
                assert int(gpu["tokens"][i][b]) == gen.tokens[i], f"token seq {b} step {i}: margin {margin:.3e}"
    return worst_logit, worst_hidden
