"""No-KV-cache brute force of D^3 decoding in NumPy float64.  TEST INFRASTRUCTURE
ONLY; it shares no code with the C oracle and exists to pin it.

Every generated token re-runs the whole sequence, block by block, with full
[S, S] causal attention matrices.  Which blocks a row runs through is decided per
row: prompt rows run every block (Section 3.1 / 3.2: the prompt pass uses all
layers); the row fed at decode step j runs the blocks the schedule keeps for
T_j (Section 3.4, Table 6).  Because the kept count never grows with j, the rows
that run block l always form a prefix of the sequence within one request, so a
row that runs block l finds the keys and values of every earlier row there (the
code asserts it).

With fill=True, a row that skipped block l instead exposes, in block l, the K/V
it produced in the last block before its drop window (the COPY policy of
Section 3.2); this is only supported for start >= 1.  With fill="recompute" it
exposes instead the K/V that block l's own projections make of the row's current
residual, i.e. of the hidden state copied through the skipped blocks (the
recompute policy of the same passage).
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Optional, Sequence

import numpy as np


def kept_blocks(L: int, alpha_decimal: str, i: int) -> int:
    """floor(L * alpha^i) in exact rational arithmetic on the decimal string of alpha."""
    v = L * Fraction(alpha_decimal) ** i
    return v.numerator // v.denominator


def executed_blocks(L: int, alpha_decimal: str, start: int, i: int, min_keep: int = 0) -> List[int]:
    k = max(min_keep, kept_blocks(L, alpha_decimal, i))
    n = L - k
    s = min(start, L - n)
    return [l for l in range(L) if not (s <= l < s + n)]


def kept_blocks_linear(L: int, keep_first: int, keep_last: int, n_steps: int, i: int) -> int:
    """floor of the straight line from keep_first (step 0) to keep_last (step n_steps - 1), in exact rationals."""
    y = Fraction(keep_first) - Fraction(keep_first - keep_last) * Fraction(i, max(1, n_steps - 1))
    return y.numerator // y.denominator


def executed_blocks_linear(L: int, keep_first: int, keep_last: int, n_steps: int, start: int, i: int) -> List[int]:
    n = L - kept_blocks_linear(L, keep_first, keep_last, n_steps, i)
    s = min(start, L - n)
    return [l for l in range(L) if not (s <= l < s + n)]


def _rms(x, gain, eps):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gain


def _rope_all(x, positions, hd, base):
    """x [S, heads, hd]; rotate pairs (j, j+hd/2) by positions * base**(-2j/hd)."""
    half = hd // 2
    inv = base ** (-np.arange(half, dtype=np.float64) * 2.0 / hd)
    ang = positions[:, None].astype(np.float64) * inv[None, :]          # [S, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def forward_all(shape, w64, tokens: Sequence[int], row_blocks: List[Sequence[int]], fill: bool = False,
                row_src: Optional[List[Optional[int]]] = None):
    """Run the whole sequence.  row_blocks[t] = blocks row t executes; with fill,
    row_src[t] = block whose K/V row t exposes in the blocks it skipped.
    Returns (logits of the last row [V], hidden of last row [(n_exec+1), d])."""
    s = shape
    S = len(tokens)
    X = w64["tok_emb"][np.asarray(tokens)].copy()                         # [S, d]
    pos = np.arange(S)
    group = s.H // s.H_kv
    last_hidden = [X[-1].copy()]
    runs = np.zeros((S, s.L), bool)
    for t, blocks in enumerate(row_blocks):
        runs[t, list(blocks)] = True
    Ks, Vs = {}, {}
    for l in range(s.L):
        act = np.nonzero(runs[:, l])[0]
        if act.size == 0:
            continue                           # (nobody reads this block's rows either)
        lw = w64["layers"][l]
        A = _rms(X[act], lw["attn_norm"], s.eps)
        Q = _rope_all((A @ lw["wq"].T).reshape(-1, s.H, s.hd), pos[act], s.hd, s.rope_base)
        K = _rope_all((A @ lw["wk"].T).reshape(-1, s.H_kv, s.hd), pos[act], s.hd, s.rope_base)
        V = (A @ lw["wv"].T).reshape(-1, s.H_kv, s.hd)
        Kf = np.zeros((S, s.H_kv, s.hd)); Vf = np.zeros((S, s.H_kv, s.hd))
        have = np.zeros(S, bool)
        Kf[act], Vf[act], have[act] = K, V, True
        if fill == "recompute":                # skipped rows expose the K/V this block makes of their copied hidden state
            idle = np.nonzero(~runs[:, l])[0]
            if idle.size:
                Ai = _rms(X[idle], lw["attn_norm"], s.eps)
                Kf[idle] = _rope_all((Ai @ lw["wk"].T).reshape(-1, s.H_kv, s.hd), pos[idle], s.hd, s.rope_base)
                Vf[idle] = (Ai @ lw["wv"].T).reshape(-1, s.H_kv, s.hd)
                have[idle] = True
        elif fill:                             # skipped rows expose their source block's K/V here
            for t in np.nonzero(~runs[:, l])[0]:
                src = row_src[t]
                assert src is not None and src < l and runs[t, src]
                Kf[t], Vf[t], have[t] = Ks[src][t], Vs[src][t], True
        Ks[l], Vs[l] = Kf, Vf
        mask = pos[None, :] <= act[:, None]                               # [n_act, S] causal
        assert have[np.nonzero(mask.any(axis=0))[0]].all(), "an executed row would read a missing K/V row"
        O = np.zeros((act.size, s.H, s.hd))
        for h in range(s.H):
            kv = h // group
            sc = Q[:, h, :] @ Kf[:, kv, :].T / np.sqrt(s.hd)
            sc = np.where(mask, sc, -np.inf)
            sc = np.exp(sc - sc.max(axis=1, keepdims=True))
            sc /= sc.sum(axis=1, keepdims=True)
            O[:, h, :] = sc @ Vf[:, kv, :]
        X[act] = X[act] + O.reshape(act.size, s.H * s.hd) @ lw["wo"].T
        M = _rms(X[act], lw["mlp_norm"], s.eps)
        gate = M @ lw["w_gate"].T
        X[act] = X[act] + (gate / (1.0 + np.exp(-gate)) * (M @ lw["w_up"].T)) @ lw["w_down"].T
        if runs[S - 1, l]:
            last_hidden.append(X[-1].copy())
    logits = _rms(X[-1], w64["final_norm"], s.eps) @ w64["lm_head"].T
    return logits, np.stack(last_hidden)


def generate(shape, w64, prompt: Sequence[int], G: int, alpha_decimal: str, start: int, min_keep: int = 0,
             forced: Optional[Sequence[int]] = None, step_blocks: Optional[Sequence[Sequence[int]]] = None):
    """Greedy D^3 generation with no cache.  Returns (tokens [G], logits [G][V], hidden list).
    step_blocks[i], if given, lists the blocks step i executes instead of the power law's."""
    P = len(prompt)
    all_blocks = list(range(shape.L))
    tokens, logits_all, hidden_all = [], [], []
    seq = list(int(t) for t in prompt)
    row_blocks = [all_blocks] * P
    for i in range(G):
        if i >= 1:
            seq.append(int(forced[i - 1]) if forced is not None else tokens[i - 1])
            row_blocks = row_blocks + [list(step_blocks[i]) if step_blocks is not None
                                       else executed_blocks(shape.L, alpha_decimal, start, i, min_keep)]
        logits, hidden = forward_all(shape, w64, seq, row_blocks)
        tokens.append(int(np.argmax(logits)))
        logits_all.append(logits)
        hidden_all.append(hidden)
    return tokens, logits_all, hidden_all
