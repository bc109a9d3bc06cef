"""GPU tests of the missing-state fill, continuation on a filled cache, and call-order checks."""
import numpy as np
import pytest

import d3_inputs
from d3_inputs import ModelShape
from oracle import oracle
from tests import helpers

pytestmark = pytest.mark.gpu

SHAPE = ModelShape("fill-bf16", L=6, d=256, H=4, H_kv=2, hd=64, F=704, V=1024, dtype="bf16")


def _cache_rows(dec, layer, seq, pos):
    """K and V of one (block, sequence, row) as float64 [H_kv*hd] (head-major, like the oracle's rows)."""
    k = dec.k_cache[layer, seq, :, pos, :].float().cpu().numpy().astype(np.float64).reshape(-1)
    v = dec.v_cache[layer, seq, :, pos, :].float().cpu().numpy().astype(np.float64).reshape(-1)
    return k, v


@pytest.mark.parametrize("start,kv", [(2, "f16"), (0, "f16"), (4, "f32")])
@pytest.mark.parametrize("lazy", [False, True])
def test_fill_copies_the_source_block_and_matches_oracle(start, kv, lazy):
    import torch
    shape, B, P, G, alpha = SHAPE, 3, 6, 9, 0.8
    w = d3_inputs.make_weights(shape, 2)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = d3_inputs.make_prompt(B, G - 1, shape.V, seed=4)
    print(f"case fill start={start} kv={kv} lazy={lazy}", flush=True)
    gpu = helpers.gpu_generate(shape, w, prompts, G, alpha, start, forced=forced, kv_dtype=kv, fill_each_step=not lazy,
                               max_seq=P + G + 8)
    dec = gpu["decoder"]
    if lazy:
        dec.fill_missing_kv(0, dec.n_ctx)            # prompt rows need nothing; generated rows filled in one call
    torch.cuda.synchronize()
    model, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced, max_seq=P + G + 8)
    L = shape.L
    tol = {"f32": 2e-5, "f16": 4e-3}[kv]
    for b, gen in enumerate(gens):
        oracle.fill_generated_rows(gen, P, G)
        for i in range(1, G):
            pos = P + i - 1
            s, n = int(gen.drop_begin[i]), L - int(gen.keep[i])
            src = s - 1 if s > 0 else s + n
            for l in range(s, s + n):
                kg, vg = _cache_rows(dec, l, b, pos)
                ks, vs = _cache_rows(dec, src, b, pos)
                assert (kg == ks).all() and (vg == vs).all()              # a copy is bit-exact
                ko, vo = gen.seq.get_kv(l, pos)
                assert np.abs(kg - ko).max() <= tol * max(1.0, np.abs(ko).max())
                assert np.abs(vg - vo).max() <= tol * max(1.0, np.abs(vo).max())
    # rows of executed blocks are untouched by the fill: compare one against the oracle too
    kg, _ = _cache_rows(dec, 0, 0, P)
    ko, _ = gens[0].seq.get_kv(0, P)
    assert np.abs(kg - ko).max() <= tol * max(1.0, np.abs(ko).max())


def test_continuation_reads_filled_rows():
    # a second request on the same cache runs at full depth again and attends to the copied K/V rows
    import torch
    from paper_2503_08524_amd import binding
    shape, B, P, G, alpha, start = SHAPE, 2, 5, 7, 0.8, 2
    P2, G2 = 4, 4
    w = d3_inputs.make_weights(shape, 3)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = d3_inputs.make_prompt(B, G - 1, shape.V, seed=4)
    prompts2 = d3_inputs.make_prompt(B, P2, shape.V, seed=5)
    forced2 = d3_inputs.make_prompt(B, G2 - 1, shape.V, seed=6)
    max_seq = P + G + P2 + G2
    print("case continuation", flush=True)
    gpu = helpers.gpu_generate(shape, w, prompts, G, alpha, start, forced=forced, max_seq=max_seq, fill_each_step=True)
    dec = gpu["decoder"]
    n_rows = P + G - 1
    assert dec.n_ctx == n_rows
    gpu2 = helpers.gpu_generate(shape, w, prompts2, G2, alpha, start, forced=forced2, decoder=dec, pos_begin=n_rows)
    model, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced, max_seq=max_seq)
    gens2 = []
    for b, gen in enumerate(gens):
        oracle.fill_generated_rows(gen, P, G)
        gens2.append(oracle.generate(model, prompts2[b], G2, alpha, start, seq=gen.seq, pos_begin=n_rows, forced=forced2[b]))
    helpers.compare(gpu, gens, G)
    wl, wh = helpers.compare(gpu2, gens2, G2)
    print(f"  continuation worst logit abs err {wl:.3e}, hidden {wh:.3e}", flush=True)


def test_call_order_and_range_errors():
    import torch
    from paper_2503_08524_amd import binding, D3Error
    shape = SHAPE
    w = binding.weights_to_device(shape, d3_inputs.make_weights(shape, 2))
    dec = binding.Decoder(shape, w, 2, 12)
    tok = torch.zeros(2, dtype=torch.int32, device="cuda:0")
    out = torch.zeros_like(tok)
    prompts = torch.from_numpy(d3_inputs.make_prompt(2, 8, shape.V, seed=1)).to("cuda:0")

    def status(fn):
        with pytest.raises(D3Error) as e:
            fn()
        return e.value.status

    assert status(lambda: dec.decode_step(tok, 1, out)) == -4                      # no plan
    dec.set_plan(0.9, 2, 0, 4)
    assert status(lambda: dec.decode_step(tok, 1, out)) == -4                      # no prompt pass
    assert status(lambda: dec.prefill(prompts[:, :0].contiguous())) == -1          # empty prompt
    assert status(lambda: dec.prefill(torch.zeros(3, 4, dtype=torch.int32, device="cuda:0"))) == -2   # batch > max_batch
    assert status(lambda: dec.prefill(torch.zeros(2, 13, dtype=torch.int32, device="cuda:0"))) == -3  # beyond max_seq
    assert status(lambda: dec.prefill(prompts, pos_begin=3)) == -4                 # neither 0 nor the row count
    assert status(lambda: dec.prefill_ragged(prompts, [0, 8])) == -1               # an empty sequence
    assert status(lambda: dec.prefill_ragged(prompts, [9, 8])) == -1               # longer than the padded width
    assert status(lambda: dec.prefill_ragged(prompts, [7, 5])) == -1               # not padded to the longest
    assert status(lambda: dec.set_plan_table([6, 7], [0, 0])) == -1                # keeps more blocks than there are
    dec.prefill_ragged(prompts, [8, 5])
    assert status(lambda: dec.truncate(3)) == -3                                   # sequence 1 begins at row 3: it would keep no row
    dec.truncate(4)
    assert dec.n_ctx == 4
    dec.prefill(prompts)
    assert dec.n_ctx == 8
    assert status(lambda: dec.decode_step(tok, 2, out)) == -4                      # steps must come in order
    dec.decode_step(tok, 1, out)
    dec.decode_step(out, 2, tok)
    dec.decode_step(tok, 3, out)
    assert status(lambda: dec.decode_step(out, 4, tok)) == -3                      # outside the plan of 4 steps
    assert status(lambda: dec.fill_missing_kv(0, 99)) == -3
    assert status(lambda: dec.fill_missing_kv(0, 4, mode=7)) == -1
    assert status(lambda: dec.truncate(0)) == -3
    assert status(lambda: dec.truncate(99)) == -3
    dec.set_plan(1.0, 2, 0, 8)
    dec.decode_step(tok, 1, out)                                                   # row 11: the last one
    assert status(lambda: dec.decode_step(out, 2, tok)) == -3                      # cache full
    dec.truncate(8)
    assert dec.n_ctx == 8
    dec.decode_step(tok, 1, out)
    torch.cuda.synchronize()
    dec.close()


def test_decode_is_deterministic_and_rewind_reproduces_it():
    import torch
    from paper_2503_08524_amd import binding
    shape = SHAPE
    w = binding.weights_to_device(shape, d3_inputs.make_weights(shape, 2))
    dec = binding.Decoder(shape, w, 2, 40)
    prompts = torch.from_numpy(d3_inputs.make_prompt(2, 20, shape.V, seed=1)).to("cuda:0")
    dec.set_plan(0.85, 2, 0, 16)
    first = dec.prefill(prompts)
    runs = []
    for _ in range(2):
        dec.truncate(20)
        dec.set_plan(0.85, 2, 0, 16)
        cur, nxt = first.clone(), torch.zeros_like(first)
        logits = torch.zeros(2, shape.V, device="cuda:0")
        rec = []
        for i in range(1, 16):
            dec.decode_step(cur, i, nxt, logits=logits)
            rec.append((nxt.cpu().numpy().copy(), logits.cpu().numpy().copy()))
            cur, nxt = nxt, cur
        runs.append(rec)
    for (t0, l0), (t1, l1) in zip(*runs):
        assert (t0 == t1).all() and (l0 == l1).all()                              # bit-identical replays


def _check_recomputed_rows(dec, gens, shape, P, G, tol, lengths=None):
    L = shape.L
    worst = 0.0
    for b, gen in enumerate(gens):
        own = P if lengths is None else int(lengths[b])      # the oracle's sequence knows nothing of its padding
        oracle.fill_generated_rows(gen, own, G, mode="recompute")
        for i in range(1, G):
            pos = P + i - 1
            s, n = int(gen.drop_begin[i]), L - int(gen.keep[i])
            for l in range(s, s + n):
                kg, vg = _cache_rows(dec, l, b, pos)
                ko, vo = gen.seq.get_kv(l, own + i - 1)
                ek = np.abs(kg - ko).max() / max(1.0, np.abs(ko).max())
                ev = np.abs(vg - vo).max() / max(1.0, np.abs(vo).max())
                worst = max(worst, ek, ev)
                assert ek <= tol and ev <= tol, f"seq {b} step {i} block {l}: K {ek:.3e} V {ev:.3e}"
    return worst


@pytest.mark.parametrize("B,start,kv", [(1, 2, "f16"), (1, 0, "f32"), (3, 2, "f16"), (3, 4, "f32"), (2, 0, "f16")])
def test_recompute_fill_matches_oracle_and_continuation_reads_it(B, start, kv):
    """RECOMPUTE fill: K/V of every dropped block recomputed from the hidden state copied through the drop window
    (batch 1: the fused QKV kernel without q heads; batch >= 2: the matrix-core path), then a second request on the
    same cache at full depth reads the recomputed rows."""
    import torch
    from paper_2503_08524_amd import binding
    shape, P, G, alpha = SHAPE, 6, 9, 0.8
    P2, G2 = 4, 4
    w = d3_inputs.make_weights(shape, 2)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = d3_inputs.make_prompt(B, G - 1, shape.V, seed=4)
    prompts2 = d3_inputs.make_prompt(B, P2, shape.V, seed=5)
    forced2 = d3_inputs.make_prompt(B, G2 - 1, shape.V, seed=6)
    max_seq = P + G + P2 + G2
    print(f"case recompute fill B={B} start={start} kv={kv}", flush=True)
    gpu = helpers.gpu_generate(shape, w, prompts, G, alpha, start, forced=forced, kv_dtype=kv, fill_each_step=True,
                               max_seq=max_seq, fill_mode=binding.D3_FILL_RECOMPUTE)
    dec = gpu["decoder"]
    torch.cuda.synchronize()
    model, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced, max_seq=max_seq)
    tol = {"f32": 5e-5, "f16": 4e-3}[kv]
    worst = _check_recomputed_rows(dec, gens, shape, P, G, tol)
    n_rows = P + G - 1
    gpu2 = helpers.gpu_generate(shape, w, prompts2, G2, alpha, start, forced=forced2, decoder=dec, pos_begin=n_rows)
    gens2 = [oracle.generate(model, prompts2[b], G2, alpha, start, seq=gen.seq, pos_begin=n_rows, forced=forced2[b])
             for b, gen in enumerate(gens)]
    wl, wh = helpers.compare(gpu2, gens2, G2)
    print(f"  worst recomputed row err {worst:.3e}; continuation logit abs err {wl:.3e}, hidden {wh:.3e}", flush=True)


@pytest.mark.parametrize("mode", ["copy", "recompute"])
def test_schedule_whose_depth_rises_again_reads_the_filled_rows(mode):
    """The case the paper's first challenge describes (Section 1): a token runs blocks that an earlier token skipped, so
    the earlier token's missing K/V rows are read within the same request.  A caller-made schedule (not nested, windows
    at different places) with the fill after every step, against the oracle stepped the same way."""
    import torch
    from paper_2503_08524_amd import binding
    shape, B, P = SHAPE, 2, 7
    L = shape.L
    keep = np.array([6, 3, 5, 2, 6, 4, 1, 6, 0, 5], np.int32)
    drop = np.array([0, 1, 0, 2, 0, 4, 1, 0, 0, 5], np.int32)
    G = len(keep)
    w = d3_inputs.make_weights(shape, 2)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = d3_inputs.make_prompt(B, G - 1, shape.V, seed=4)
    fm = binding.D3_FILL_RECOMPUTE if mode == "recompute" else binding.D3_FILL_COPY
    print(f"case rising depth, fill {mode}", flush=True)
    dec = binding.Decoder(shape, binding.weights_to_device(shape, w), B, P + G, kv_dtype="f16")
    dec.set_plan_table(keep, drop)
    dec.set_fill_mode(fm)
    dev = "cuda:0"
    logits = torch.zeros(B, shape.V, device=dev)
    cur = dec.prefill(torch.from_numpy(prompts).to(dev), logits=logits)
    got = [logits.cpu().numpy().copy()]
    nxt = torch.zeros_like(cur)
    for i in range(1, G):
        cur = torch.from_numpy(np.ascontiguousarray(forced[:, i - 1], np.int32)).to(dev)
        dec.decode_step(cur, i, nxt, logits=logits)
        dec.fill_missing_kv(dec.n_ctx - 1, dec.n_ctx, fm)
        got.append(logits.cpu().numpy().copy())
    dec.synchronize()
    ids = binding.d3_plan_from_table(L, keep, drop)
    oracle.set_threads(helpers.oracle_threads())
    model = oracle.OracleModel(shape, w)
    worst = 0.0
    for b in range(B):
        seq = model.new_seq(P + G)
        for t in range(P):
            _, lg = seq.forward_token(int(prompts[b, t]), t, list(range(L)), False, t == P - 1)
        worst = max(worst, float(np.abs(got[0][b] - lg).max()))
        for i in range(1, G):
            blocks = ids[i, : keep[i]]
            hid, lg = seq.forward_token(int(forced[b, i - 1]), P + i - 1, blocks, True, True)
            if mode == "copy":
                seq.fill_missing_kv(P + i - 1, int(drop[i]), int(L - keep[i]))
            else:
                seq.fill_recompute(P + i - 1, int(drop[i]), int(L - keep[i]), hid[int((blocks < drop[i]).sum())])
            worst = max(worst, float(np.abs(got[i][b] - lg).max()))
    print(f"  worst logit abs err {worst:.3e}", flush=True)
    assert worst <= helpers.LOGIT_ATOL
    dec.close()


@pytest.mark.parametrize("mode", ["copy", "recompute"])
def test_left_padded_batch_fill_and_continuation(mode):
    """A ragged batch: the fill of each sequence's dropped blocks and a second request on the same cache (equal tails)
    against per-sequence oracles that know nothing of the padding."""
    import torch
    from paper_2503_08524_amd import binding
    shape, alpha, start, kv = SHAPE, 0.8, 2, "f16"
    lengths = np.array([6, 2, 5], np.int32)
    B, P, G, P2, G2 = 3, 6, 9, 4, 4
    w = d3_inputs.make_weights(shape, 2)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = d3_inputs.make_prompt(B, G - 1, shape.V, seed=4)
    prompts2 = d3_inputs.make_prompt(B, P2, shape.V, seed=5)
    forced2 = d3_inputs.make_prompt(B, G2 - 1, shape.V, seed=6)
    max_seq = P + G + P2 + G2
    print(f"case ragged fill {mode}", flush=True)
    fm = binding.D3_FILL_RECOMPUTE if mode == "recompute" else binding.D3_FILL_COPY
    gpu = helpers.gpu_generate(shape, w, prompts, G, alpha, start, forced=forced, kv_dtype=kv, fill_each_step=True,
                               max_seq=max_seq, fill_mode=fm, lengths=lengths)
    dec = gpu["decoder"]
    torch.cuda.synchronize()
    model, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced, max_seq=max_seq, lengths=lengths)
    helpers.compare(gpu, gens, G)
    if mode == "recompute":
        _check_recomputed_rows(dec, gens, shape, P, G, 4e-3, lengths=lengths)
    else:
        for b, gen in enumerate(gens):
            oracle.fill_generated_rows(gen, int(lengths[b]), G)
    gpu2 = helpers.gpu_generate(shape, w, prompts2, G2, alpha, start, forced=forced2, decoder=dec, pos_begin=P + G - 1)
    gens2 = [oracle.generate(model, prompts2[b], G2, alpha, start, seq=gen.seq, pos_begin=int(lengths[b]) + G - 1, forced=forced2[b])
             for b, gen in enumerate(gens)]
    wl, wh = helpers.compare(gpu2, gens2, G2)
    print(f"  continuation logit abs err {wl:.3e}, hidden {wh:.3e}", flush=True)


@pytest.mark.parametrize("name,B", [("llama-7b", 1), ("llama-70b", 2)])
def test_recompute_fill_at_real_widths(name, B):
    import torch
    from paper_2503_08524_amd import binding
    shape = d3_inputs.SHAPES[name].truncated(3)
    P, G, alpha, start = 24, 4, 0.6, 1                  # keeps 3, 1, 1, 0 blocks: windows [1,3), [1,3), [0,3)
    w = d3_inputs.make_weights(shape, 0)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = d3_inputs.make_prompt(B, G - 1, shape.V, seed=4)
    print(f"case recompute fill {shape.name} B={B}", flush=True)
    gpu = helpers.gpu_generate(shape, w, prompts, G, alpha, start, forced=forced, fill_each_step=True,
                               fill_mode=binding.D3_FILL_RECOMPUTE)
    torch.cuda.synchronize()
    model, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced)
    assert [int(k) for k in gens[0].keep[:G]] == [3, 1, 1, 0]
    worst = _check_recomputed_rows(gpu["decoder"], gens, shape, P, G, 4e-3)
    print(f"  worst recomputed row err {worst:.3e}", flush=True)


def test_recompute_fill_call_rules():
    import torch
    from paper_2503_08524_amd import binding, D3Error
    shape = SHAPE
    w = binding.weights_to_device(shape, d3_inputs.make_weights(shape, 2))
    dec = binding.Decoder(shape, w, 2, 16)
    prompts = torch.from_numpy(d3_inputs.make_prompt(2, 6, shape.V, seed=1)).to("cuda:0")
    tok = torch.zeros(2, dtype=torch.int32, device="cuda:0")
    out = torch.zeros_like(tok)

    def status(fn):
        with pytest.raises(D3Error) as e:
            fn()
        return e.value.status

    dec.set_plan(0.7, 2, 0, 6)
    dec.prefill(prompts)
    dec.decode_step(tok, 1, out)
    assert status(lambda: dec.fill_missing_kv(6, 7, binding.D3_FILL_RECOMPUTE)) == -4    # mode was not declared before the step
    assert status(lambda: dec.set_fill_mode(7)) == -1
    dec.set_fill_mode(binding.D3_FILL_RECOMPUTE)
    assert status(lambda: dec.fill_missing_kv(6, 7, binding.D3_FILL_RECOMPUTE)) == -4    # that step kept no residual
    dec.decode_step(tok, 2, out)
    assert status(lambda: dec.fill_missing_kv(6, 8, binding.D3_FILL_RECOMPUTE)) == -4    # only the latest row
    assert status(lambda: dec.fill_missing_kv(6, 7, binding.D3_FILL_RECOMPUTE)) == -4
    dec.fill_missing_kv(7, 8, binding.D3_FILL_RECOMPUTE)
    dec.fill_missing_kv(6, 7, binding.D3_FILL_COPY)                                     # COPY stays available for any row
    dec.synchronize()
    dec.close()


@pytest.mark.parametrize("P2", [10, 150])
def test_continuation_prompt_whose_query_tiles_straddle_an_attention_split(P2):
    """A second prompt that starts at row 125: its chunk's query tiles (4 queries x 4 heads of a KV head at this shape) are
    not aligned with the context splits (multiples of 64 rows, 128 by default), so some queries of a tile have no row in
    the last split while others do."""
    shape = ModelShape("small-gqa", L=3, d=512, H=8, H_kv=2, hd=128, F=1376, V=2000, dtype="bf16")
    B, P, G, alpha, start = 2, 114, 12, 0.9, 1
    G2 = 3                                             # P2 = 150: a full 128-column chunk and a remainder, both on a cache that already holds rows
    w = d3_inputs.make_weights(shape, 3)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = d3_inputs.make_prompt(B, G - 1, shape.V, seed=4)
    prompts2 = d3_inputs.make_prompt(B, P2, shape.V, seed=5)
    forced2 = d3_inputs.make_prompt(B, G2 - 1, shape.V, seed=6)
    max_seq = P + G + P2 + G2
    print("case continuation across a split boundary", flush=True)
    gpu = helpers.gpu_generate(shape, w, prompts, G, alpha, start, forced=forced, max_seq=max_seq, fill_each_step=True)
    dec = gpu["decoder"]
    n_rows = P + G - 1
    assert n_rows == 125
    gpu2 = helpers.gpu_generate(shape, w, prompts2, G2, alpha, start, forced=forced2, decoder=dec, pos_begin=n_rows)
    model, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced, max_seq=max_seq)
    gens2 = []
    for b, gen in enumerate(gens):
        oracle.fill_generated_rows(gen, P, G)
        gens2.append(oracle.generate(model, prompts2[b], G2, alpha, start, seq=gen.seq, pos_begin=n_rows, forced=forced2[b]))
    wl, wh = helpers.compare(gpu2, gens2, G2)
    print(f"  worst logit abs err {wl:.3e}, hidden {wh:.3e}", flush=True)


def test_measurement_aids_run_and_check_their_arguments():
    # the read-only stream and the matrix-core yardstick that bench.py holds its rates against: every mode runs to the
    # end on a small model's workspace, bad arguments are refused before anything is launched
    import torch
    from paper_2503_08524_amd import binding, D3Error
    shape = SHAPE
    w = binding.weights_to_device(shape, d3_inputs.make_weights(shape, 2))
    dec = binding.Decoder(shape, w, 1, 16)
    for mode in (0, 1, 2):
        dec.mfma_yardstick(mode, 64)
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    dec.stream_read(buf)
    torch.cuda.synchronize()
    for mode, stages in ((3, 64), (-1, 64), (0, 0), (0, 63), (0, (1 << 20) + 2)):
        with pytest.raises(D3Error) as e:
            dec.mfma_yardstick(mode, stages)
        assert e.value.status == -1
    with pytest.raises(D3Error) as e:
        dec.stream_read(buf[1:17])
    assert e.value.status == -1
    dec.close()
