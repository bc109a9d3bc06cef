"""Pins of the oracle's decoder arithmetic (no GPU).

The C oracle is checked against things that are not itself: a NumPy brute force
with no KV cache (separately written), torch's CPU library routines for one
decoder block, and closed forms / invariants of the sub-functions.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as Fn

import d3_inputs
from d3_inputs import ModelShape
from oracle import bruteforce, oracle

MICRO = ModelShape("micro", L=5, d=48, H=6, H_kv=6, hd=8, F=80, V=64, dtype="f32")
MICRO_GQA = ModelShape("micro-gqa", L=6, d=64, H=8, H_kv=2, hd=16, F=96, V=50, dtype="bf16")


def _setup(shape, seed=0):
    w = d3_inputs.make_weights(shape, seed)
    return w, d3_inputs.weights_as_f64(shape, w), oracle.OracleModel(shape, w)


# ---------- whole-path pins: C oracle (KV cache) vs NumPy brute force (no cache) ----------

@pytest.mark.parametrize("shape,alpha,start", [
    (MICRO, "1.0", 2), (MICRO, "0.9", 2), (MICRO, "0.8", 1), (MICRO, "0.9", 4), (MICRO, "0.85", 0),
    (MICRO_GQA, "0.93", 3), (MICRO_GQA, "1.0", 3), (d3_inputs.TINY.truncated(3), "0.8", 1),
])
def test_oracle_matches_no_cache_brute_force(shape, alpha, start):
    w, w64, model = _setup(shape)
    P, G = 7, 9
    prompt = d3_inputs.make_prompt(1, P, shape.V, seed=3)[0]
    gen = oracle.generate(model, prompt, G, float(alpha), start)
    # teacher-force the brute force with the oracle's tokens so one near-tie cannot cascade
    toks, logits, hidden = bruteforce.generate(shape, w64, prompt, G, alpha, start, forced=gen.tokens)
    for i in range(G):
        np.testing.assert_allclose(gen.logits[i], logits[i], rtol=0, atol=1e-11)
        np.testing.assert_allclose(gen.hidden[i], hidden[i], rtol=0, atol=1e-11)
        margin = np.sort(gen.logits[i])[-1] - np.sort(gen.logits[i])[-2]
        if margin > 1e-9:
            assert toks[i] == gen.tokens[i]
    assert [h.shape[0] - 1 for h in gen.hidden] == gen.keep[:G].tolist()


def test_alpha_one_is_plain_full_depth_decoding():
    shape = MICRO
    w, w64, model = _setup(shape, seed=5)
    prompt = d3_inputs.make_prompt(1, 6, shape.V, seed=2)[0]
    gen = oracle.generate(model, prompt, 6, 1.0, 2)
    assert (gen.keep == shape.L).all()
    # textbook decoder: every row through every block, no schedule involved at all
    seq = list(prompt)
    for i in range(6):
        logits, _ = bruteforce.forward_all(shape, w64, seq, [range(shape.L)] * len(seq))
        np.testing.assert_allclose(gen.logits[i], logits, rtol=0, atol=1e-11)
        seq.append(gen.tokens[i])


def test_skipped_blocks_leave_hidden_and_cache_untouched():
    shape = MICRO
    w, w64, model = _setup(shape)
    seq = model.new_seq(8)
    seq.forward_token(3, 0, [0, 1, 2, 3, 4])
    hid, _ = seq.forward_token(5, 1, [0, 4], want_hidden=True)
    assert hid.shape == (3, shape.d)
    for l in (1, 2, 3):
        k, v = seq.get_kv(l, 1)
        assert not k.any() and not v.any()          # rows of skipped blocks are never written
    for l in (0, 4):
        k, v = seq.get_kv(l, 1)
        assert k.any() and v.any()


def test_fill_is_a_copy_and_continuation_matches_brute_force():
    shape, alpha, start = MICRO, "0.8", 2
    w, w64, model = _setup(shape, seed=7)
    P, G, P2, G2 = 5, 6, 3, 3
    prompt = d3_inputs.make_prompt(1, P, shape.V, seed=4)[0]
    gen = oracle.generate(model, prompt, G, float(alpha), start, max_seq=P + G + P2 + G2)
    oracle.fill_generated_rows(gen, P, G)
    L = shape.L
    row_blocks = [list(range(L))] * P
    row_src = [None] * P
    for i in range(1, G):
        pos = P + i - 1
        n, s = L - gen.keep[i], gen.drop_begin[i]
        for l in range(s, s + n):                    # definitional: bitwise copy of the source block's row
            assert all((a == b).all() for a, b in zip(seq_kv(gen, l, pos), seq_kv(gen, s - 1, pos)))
        row_blocks.append(bruteforce.executed_blocks(L, alpha, start, i))
        row_src.append(int(s) - 1)
    # continuation: a second request on the same cache runs full depth again and reads the filled rows
    prompt2 = d3_inputs.make_prompt(1, P2, shape.V, seed=9)[0]
    n_rows = P + G - 1
    gen2 = oracle.generate(model, prompt2, G2, float(alpha), start, seq=gen.seq, pos_begin=n_rows)
    tokens = list(prompt) + gen.tokens[:G - 1] + list(prompt2)
    row_blocks += [list(range(L))] * P2
    row_src += [None] * P2
    for i in range(G2):
        if i >= 1:
            tokens.append(gen2.tokens[i - 1])
            row_blocks.append(bruteforce.executed_blocks(L, alpha, start, i))
            row_src.append(int(gen2.drop_begin[i]) - 1)
        logits, _ = bruteforce.forward_all(shape, w64, tokens, row_blocks, fill=True, row_src=row_src)
        np.testing.assert_allclose(gen2.logits[i], logits, rtol=0, atol=1e-11)


def seq_kv(gen, layer, pos):
    return gen.seq.get_kv(layer, pos)


def test_fill_source_when_window_starts_at_block_zero_and_when_nothing_ran():
    shape = MICRO
    _, _, model = _setup(shape)
    seq = model.new_seq(4)
    seq.forward_token(1, 0, [3, 4])                  # blocks 0..2 dropped: source is block 3
    seq.fill_missing_kv(0, 0, 3)
    for l in range(3):
        assert (seq.get_kv(l, 0)[0] == seq.get_kv(3, 0)[0]).all() and (seq.get_kv(l, 0)[1] == seq.get_kv(3, 0)[1]).all()
    seq.forward_token(1, 1, [0, 1, 2, 3, 4])
    seq.fill_missing_kv(1, 0, 5)                     # pretend no block ran: zero fill
    assert not any(seq.get_kv(l, 1)[0].any() for l in range(5))


# ---------- one block against torch CPU library routines ----------

def test_one_block_matches_torch_library_routines():
    shape = ModelShape("one", L=1, d=64, H=8, H_kv=4, hd=8, F=112, V=40, dtype="f32")
    w, w64, model = _setup(shape, seed=11)
    S = 9
    tokens = d3_inputs.make_prompt(1, S, shape.V, seed=6)[0]
    seq = model.new_seq(S)
    got = np.stack([seq.forward_token(int(t), p, [0], want_hidden=True)[0][1] for p, t in enumerate(tokens)])

    lw = {k: torch.from_numpy(v) for k, v in w64["layers"][0].items()}
    x = torch.from_numpy(w64["tok_emb"])[torch.from_numpy(tokens.astype(np.int64))]
    a = Fn.rms_norm(x, (shape.d,), lw["attn_norm"], eps=shape.eps)
    q = Fn.linear(a, lw["wq"]).view(S, shape.H, shape.hd).transpose(0, 1)
    k = Fn.linear(a, lw["wk"]).view(S, shape.H_kv, shape.hd).transpose(0, 1)
    v = Fn.linear(a, lw["wv"]).view(S, shape.H_kv, shape.hd).transpose(0, 1)
    # rotary embedding as a complex multiplication of (first half + i * second half)
    inv = shape.rope_base ** (-torch.arange(shape.hd // 2, dtype=torch.float64) * 2 / shape.hd)
    rot = torch.polar(torch.ones(S, shape.hd // 2, dtype=torch.float64), torch.arange(S, dtype=torch.float64)[:, None] * inv)
    def rope(t):
        z = torch.complex(t[..., : shape.hd // 2], t[..., shape.hd // 2:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)
    q, k = rope(q), rope(k)
    k = k.repeat_interleave(shape.H // shape.H_kv, dim=0)
    v = v.repeat_interleave(shape.H // shape.H_kv, dim=0)
    o = Fn.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0].transpose(0, 1).reshape(S, -1)
    x = x + Fn.linear(o, lw["wo"])
    m = Fn.rms_norm(x, (shape.d,), lw["mlp_norm"], eps=shape.eps)
    x = x + Fn.linear(Fn.silu(Fn.linear(m, lw["w_gate"])) * Fn.linear(m, lw["w_up"]), lw["w_down"])
    np.testing.assert_allclose(got, x.numpy(), rtol=0, atol=1e-12)


# ---------- sub-function pins ----------

def test_rope_closed_forms():
    # hd = 2 is a plain 2-D rotation by `pos` radians
    np.testing.assert_allclose(oracle.rope([1.0, 0.0], 3, 10000.0), [math.cos(3), math.sin(3)], atol=1e-15)
    np.testing.assert_allclose(oracle.rope([0.0, 1.0], 1, 10000.0), [-math.sin(1), math.cos(1)], atol=1e-15)
    rng = np.random.default_rng(0)
    v = rng.standard_normal(64)
    assert (oracle.rope(v, 0, 10000.0) == v).all()                                   # position 0: identity
    r = oracle.rope(v, 777, 10000.0)
    assert abs(np.linalg.norm(r) - np.linalg.norm(v)) < 1e-12                        # rotation keeps the norm
    # the pair (j, j+hd/2) turns by pos * base^(-2j/hd): slowest pair of hd=64 at base 10000
    e = np.zeros(64); e[31] = 1.0
    ang = 5 * 10000.0 ** (-62 / 64)
    out = oracle.rope(e, 5, 10000.0)
    np.testing.assert_allclose([out[31], out[63]], [math.cos(ang), math.sin(ang)], atol=1e-15)
    # scores depend on the position difference only
    q, k = rng.standard_normal(64), rng.standard_normal(64)
    a = oracle.rope(q, 40, 10000.0) @ oracle.rope(k, 33, 10000.0)
    b = oracle.rope(q, 107, 10000.0) @ oracle.rope(k, 100, 10000.0)
    assert abs(a - b) < 1e-11


def test_softmax_rmsnorm_silu_closed_forms():
    p = oracle.softmax([0.0, math.log(2.0), math.log(5.0)])
    np.testing.assert_allclose(p, [1 / 8, 2 / 8, 5 / 8], atol=1e-15)
    big = oracle.softmax([1000.0, 1000.0, -1000.0])                                   # no overflow
    np.testing.assert_allclose(big, [0.5, 0.5, 0.0], atol=1e-15)
    x = np.array([3.0, -4.0, 0.0, 0.0])
    np.testing.assert_allclose(oracle.rmsnorm(x, np.ones(4), 0.0), x / 2.5, atol=1e-15)   # rms = sqrt(25/4)
    np.testing.assert_allclose(oracle.rmsnorm(x, [2, 1, 1, 1], 0.0)[0], 2 * 3 / 2.5, atol=1e-15)
    np.testing.assert_allclose(oracle.rmsnorm(x, np.ones(4), 2.75), x / 3.0, atol=1e-15)  # eps inside the root
    y = oracle.rmsnorm(np.random.default_rng(1).standard_normal(256), np.ones(256), 0.0)
    assert abs(np.mean(y * y) - 1.0) < 1e-12
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(oracle.silu(1.0) - oracle.silu(-1.0) - 1.0) < 1e-15                    # x*s(x) - (-x)*s(-x) = x
    assert abs(oracle.silu(40.0) - 40.0) < 1e-12 and abs(oracle.silu(-40.0)) < 1e-12


def test_attention_head_special_cases():
    rng = np.random.default_rng(2)
    hd, n = 16, 11
    V = rng.standard_normal((n, hd))
    q = rng.standard_normal(hd)
    # identical keys: uniform weights, output is the mean of the values
    K = np.tile(rng.standard_normal(hd), (n, 1))
    np.testing.assert_allclose(oracle.attention_head(q, K, V), V.mean(axis=0), atol=1e-13)
    # one key hugely aligned with q: output is that row of V
    K = rng.standard_normal((n, hd)); K[4] = 1e3 * q
    np.testing.assert_allclose(oracle.attention_head(q, K, V), V[4], atol=1e-9)
    # single row: output is V[0] whatever q is
    np.testing.assert_allclose(oracle.attention_head(q, K[:1], V[:1]), V[0], atol=1e-15)
    # scale is 1/sqrt(hd): two keys with scores a, b -> weights softmax([a, b] / sqrt(hd))
    K2 = np.zeros((2, hd)); K2[0, 0], K2[1, 0] = 2.0, -1.0
    q2 = np.zeros(hd); q2[0] = 4.0
    w0 = 1 / (1 + math.exp(-(8 + 4) / math.sqrt(hd)))
    np.testing.assert_allclose(oracle.attention_head(q2, K2, V[:2]), w0 * V[0] + (1 - w0) * V[1], atol=1e-14)


def test_argmax_takes_lowest_index_on_ties():
    assert oracle.argmax(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    assert oracle.argmax(np.array([-1.0, -1.0])) == 0


def test_float32_build_agrees_with_float64_build():
    shape = d3_inputs.TINY
    w = d3_inputs.make_weights(shape, 0)
    prompt = d3_inputs.make_prompt(1, 16, shape.V, seed=1)[0]
    g64 = oracle.generate(oracle.OracleModel(shape, w, "f64"), prompt, 8, 0.97, 2)
    g32 = oracle.generate(oracle.OracleModel(shape, w, "f32"), prompt, 8, 0.97, 2, forced=g64.tokens)
    for a, b in zip(g64.logits, g32.logits):
        assert np.abs(a - b).max() < 2e-5
    assert oracle._lib("f32").d3o_real_size() == 4 and oracle._lib("f64").d3o_real_size() == 8


def test_threads_do_not_change_results():
    shape = MICRO_GQA
    w, _, model = _setup(shape)
    prompt = d3_inputs.make_prompt(1, 5, shape.V, seed=1)[0]
    oracle.set_threads(1)
    a = oracle.generate(model, prompt, 4, 0.9, 3)
    oracle.set_threads(4)
    b = oracle.generate(model, prompt, 4, 0.9, 3)
    oracle.set_threads(1)
    assert all((x == y).all() for x, y in zip(a.logits, b.logits))


def test_first_block_cache_write_alone_equals_the_full_forward():
    """d3o_first_block_kv writes exactly the K/V row that forward_token writes for the first listed block (bitwise),
    and nothing else; the brute force agrees with both."""
    shape = d3_inputs.TINY
    w = d3_inputs.make_weights(shape, 3)
    model = oracle.OracleModel(shape, w)
    toks = d3_inputs.make_prompt(1, 5, shape.V, seed=9)[0]
    full, only = model.new_seq(8), model.new_seq(8)
    for layer in (0, 2):
        for p, t in enumerate(toks):
            full.forward_token(int(t), p, [layer, 3] if layer < 3 else [layer])
            only.first_block_kv(int(t), p, layer)
            kf, vf = full.get_kv(layer, p)
            ko, vo = only.get_kv(layer, p)
            assert np.array_equal(kf, ko) and np.array_equal(vf, vo)
            k3, v3 = only.get_kv(3, p)
            assert not k3.any() and not v3.any()          # no other block's row was touched


@pytest.mark.parametrize("shape,alpha,start", [(MICRO, "0.8", 2), (MICRO_GQA, "0.85", 0), (MICRO, "0.9", 4)])
def test_recompute_fill_definition_and_continuation_match_brute_force(shape, alpha, start):
    """RECOMPUTE fill (Section 3.2: copied hidden state, recomputed KV).  Definitional pin: the first block of a drop
    window sees exactly the copied state, so its recomputed row equals, bit for bit, the row the same block writes when
    it is executed right after the same predecessors.  Whole-path pin: a second request on the filled cache runs full
    depth and reads every filled row; the NumPy brute force (no cache, its own recompute code) must agree."""
    w, w64, model = _setup(shape, seed=5)
    L = shape.L
    P, G, P2, G2 = 5, 6, 3, 3
    prompt = d3_inputs.make_prompt(1, P, shape.V, seed=4)[0]
    gen = oracle.generate(model, prompt, G, float(alpha), start, max_seq=P + G + P2 + G2)
    oracle.fill_generated_rows(gen, P, G, mode="recompute")
    row_blocks = [list(range(L))] * P
    for i in range(1, G):
        pos, s, n = P + i - 1, int(gen.drop_begin[i]), int(L - gen.keep[i])
        row_blocks.append(bruteforce.executed_blocks(L, alpha, start, i))
        if n == 0:
            continue
        # a fresh cache with the same earlier rows, where row pos runs the predecessors AND block s
        ref = model.new_seq(P + G)
        for t in range(pos):
            fed = int(prompt[t]) if t < P else gen.fed[t - P]
            ref.forward_token(fed, t, row_blocks[t])
        ref.forward_token(gen.fed[i - 1], pos, [l for l in range(L) if l < s] + [s])
        kr, vr = ref.get_kv(s, pos)
        kf, vf = gen.seq.get_kv(s, pos)
        assert np.array_equal(kr, kf) and np.array_equal(vr, vf)
        if n > 1:                                    # deeper blocks of the window see the copied state, not block s's output
            assert not np.array_equal(gen.seq.get_kv(s + 1, pos)[0], kf)
    prompt2 = d3_inputs.make_prompt(1, P2, shape.V, seed=9)[0]
    gen2 = oracle.generate(model, prompt2, G2, float(alpha), start, seq=gen.seq, pos_begin=P + G - 1)
    tokens = list(prompt) + gen.tokens[:G - 1] + list(prompt2)
    row_blocks += [list(range(L))] * P2
    for i in range(G2):
        if i >= 1:
            tokens.append(gen2.tokens[i - 1])
            row_blocks.append(bruteforce.executed_blocks(L, alpha, start, i))
        logits, _ = bruteforce.forward_all(shape, w64, tokens, row_blocks, fill="recompute")
        np.testing.assert_allclose(gen2.logits[i], logits, rtol=0, atol=1e-11)


@pytest.mark.parametrize("start", [0, 2, 4])
def test_oracle_follows_a_linear_plan_like_the_no_cache_brute_force(start):
    # a schedule other than the power law (linear decay; shallow-first, middle-first and deep-first windows) goes through
    # the same cache logic: the blocks a step skipped stay out of every later row's attention
    shape = MICRO
    w, w64, model = _setup(shape)
    P, G = 6, 9
    prompt = d3_inputs.make_prompt(1, P, shape.V, seed=5)[0]
    plan = oracle.plan_depth_linear(shape.L, shape.L, 1, start, G)
    gen = oracle.generate(model, prompt, G, 1.0, 0, plan=plan)
    blocks = [bruteforce.executed_blocks_linear(shape.L, shape.L, 1, G, start, i) for i in range(G)]
    toks, logits, hidden = bruteforce.generate(shape, w64, prompt, G, "1.0", 0, forced=gen.tokens, step_blocks=blocks)
    for i in range(G):
        np.testing.assert_allclose(gen.logits[i], logits[i], rtol=0, atol=1e-11)
        np.testing.assert_allclose(gen.hidden[i], hidden[i], rtol=0, atol=1e-11)
    assert [h.shape[0] - 1 for h in gen.hidden] == plan[0][:G].tolist()


@pytest.mark.parametrize("mode", ["copy", "recompute"])
def test_rising_depth_with_fill_every_step_matches_brute_force(mode):
    # Section 1, first challenge: a token runs blocks that an earlier token skipped and reads that token's filled rows
    # inside the same request.  The oracle, stepped with a caller-made schedule and the fill after every step, against the
    # no-cache brute force in which a skipped row exposes its source block's K/V (copy) or the K/V of its copied hidden
    # state (recompute).
    shape = MICRO
    L = shape.L
    w, w64, model = _setup(shape, seed=11)
    P = 4
    keep = [5, 2, 4, 1, 5, 3, 5]
    drop = [0, 1, 1, 1, 0, 2, 0]
    prompt = d3_inputs.make_prompt(1, P, shape.V, seed=6)[0]
    fed = d3_inputs.make_prompt(1, len(keep) - 1, shape.V, seed=8)[0]
    seq = model.new_seq(P + len(keep))
    for t in range(P):
        seq.forward_token(int(prompt[t]), t, list(range(L)))
    tokens = [int(t) for t in prompt]
    row_blocks = [list(range(L))] * P
    row_src = [None] * P
    for i in range(1, len(keep)):
        n = L - keep[i]
        blocks = [l for l in range(L) if not (drop[i] <= l < drop[i] + n)]
        hid, logits = seq.forward_token(int(fed[i - 1]), P + i - 1, blocks, True, True)
        tokens.append(int(fed[i - 1]))
        row_blocks.append(blocks)
        row_src.append(drop[i] - 1 if n else None)
        want, _ = bruteforce.forward_all(shape, w64, tokens, row_blocks, fill=True if mode == "copy" else "recompute", row_src=row_src)
        np.testing.assert_allclose(logits, want, rtol=0, atol=1e-11)
        if mode == "copy":
            seq.fill_missing_kv(P + i - 1, drop[i], n)
        else:
            seq.fill_recompute(P + i - 1, drop[i], n, hid[sum(1 for l in blocks if l < drop[i])])
