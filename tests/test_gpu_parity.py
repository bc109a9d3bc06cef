"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs, element by element.  Bars: schedule bit-exact (tests/test_abi.py), logits within
2e-2 max abs, hidden state within 1e-2 relative L2 after every executed block, greedy tokens
identical on the small configurations."""
import numpy as np
import pytest

import d3_inputs
from d3_inputs import ModelShape
from tests import helpers

pytestmark = pytest.mark.gpu

# small shapes that still span several tiles and ragged tails of every kernel
SMALL_BF16 = ModelShape("small-bf16", L=4, d=256, H=4, H_kv=4, hd=64, F=704, V=1024, dtype="bf16")
SMALL_GQA = ModelShape("small-gqa", L=3, d=512, H=8, H_kv=2, hd=128, F=1376, V=2000, dtype="bf16")


def _forced(B, G, V, seed):
    return d3_inputs.make_prompt(B, max(G - 1, 1), V, seed=seed)


def _run(shape, B, P, G, alpha, start, kv_dtype=None, forced_seed=None, check_tokens="margin", seed=0, **kw):
    w = d3_inputs.make_weights(shape, seed)
    prompts = d3_inputs.make_prompt(B, P, shape.V, seed=1)
    forced = None if forced_seed is None else _forced(B, G, shape.V, forced_seed)
    print(f"case {shape.name} B={B} P={P} G={G} alpha={alpha} start={start} kv={kv_dtype}", flush=True)
    gpu = helpers.gpu_generate(shape, w, prompts, G, alpha, start, forced=forced, kv_dtype=kv_dtype, **kw)
    _, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced, min_keep=kw.get("min_keep", 0),
                                      linear=kw.get("linear"), lengths=kw.get("lengths"))
    wl, wh = helpers.compare(gpu, gens, G, check_tokens=check_tokens)
    print(f"  worst logit abs err {wl:.3e}, worst hidden rel L2 {wh:.3e}", flush=True)
    return gpu, gens


@pytest.mark.parametrize("alpha", [0.97, 1.0])
def test_tiny_config_tokens_logits_hidden(alpha):
    # the first benchmark configuration in full: fp32 weights, fp32 cache, free-running greedy decoding
    gpu, gens = _run(d3_inputs.TINY, 1, 16, 32, alpha, 2, kv_dtype="f32", check_tokens="all")
    helpers.compare(gpu, gens, 32, check_tokens="all", logit_atol=1e-4, hidden_tol=1e-5)


@pytest.mark.parametrize("start", [0, 2, 3])
def test_tiny_config_linear_decay_shallow_middle_and_deep_first(start):
    # the comparison schedules (linear decay; windows that grow from the first block, the middle, the last block)
    # are plans for the same kernels: free-running greedy decoding, tokens identical
    gpu, gens = _run(d3_inputs.TINY, 1, 16, 32, 1.0, start, kv_dtype="f32", check_tokens="all", linear=(4, 1))
    helpers.compare(gpu, gens, 32, check_tokens="all", logit_atol=1e-4, hidden_tol=1e-5)
    assert [h.shape[0] - 1 for h in gpu["hidden"][1:]] == gens[0].keep[1:32].tolist()


def test_batched_linear_decay_on_the_matrix_cores():
    gpu, gens = _run(SMALL_GQA, 5, 21, 12, 1.0, 0, forced_seed=3, linear=(3, 1))
    gpu, gens = _run(SMALL_BF16, 17, 9, 10, 1.0, 3, forced_seed=4, linear=(4, 0))


@pytest.mark.parametrize("shape,lengths,kv", [
    (d3_inputs.TINY, (16, 5, 11), "f32"),                 # fp32 weights: vector-ALU projections, one column per launch group
    (SMALL_BF16, (9, 70, 1, 33, 64), None),               # head_dim 64: vector-ALU attention; chunks of 64 + 6 columns
    (SMALL_GQA, (130, 17, 77, 130), "f16"),               # head_dim 128, f16 cache: query tiles in the prompt, MFMA attention in decode
    (SMALL_GQA, (40, 3), "f32"),
])
def test_left_padded_batch_of_unequal_prompts(shape, lengths, kv):
    # every sequence of a ragged batch must behave as if it had run alone: its own positions, its own context
    B, P = len(lengths), max(lengths)
    _run(shape, B, P, 9, 0.8, 1, kv_dtype=kv, forced_seed=21, lengths=np.array(lengths, np.int32), max_seq=P + 9)


def test_left_padded_batch_spans_attention_splits():
    # the short sequence's rows begin inside a later split: the splits below it hold nothing of it
    lengths = np.array([700, 150, 699], np.int32)
    _run(SMALL_GQA, 3, 700, 6, 0.7, 1, forced_seed=22, lengths=lengths)
    _run(SMALL_BF16, 2, 650, 4, 0.9, 2, forced_seed=23, lengths=np.array([40, 650], np.int32))


def test_bf16_shape_that_does_not_fit_the_matrix_core_tiles():
    # d_model, d_ffn not multiples of 32, vocab not a multiple of 16: batched passes stay on the vector-ALU projections
    shape = ModelShape("odd-bf16", L=3, d=264, H=4, H_kv=2, hd=64, F=696, V=1000, dtype="bf16")
    _run(shape, 3, 21, 7, 0.8, 1, forced_seed=31)
    _run(shape, 5, 40, 5, 0.8, 0, forced_seed=32, lengths=np.array([40, 7, 33, 1, 40], np.int32))


def test_tiny_config_f16_cache():
    _run(d3_inputs.TINY, 1, 16, 32, 0.97, 2, kv_dtype="f16", forced_seed=5)


def test_bf16_cache_is_refused():
    # its 8-bit mantissa puts the logits outside the tolerance after two blocks at real widths
    from paper_2503_08524_amd import binding
    w = binding.weights_to_device(SMALL_BF16, d3_inputs.make_weights(SMALL_BF16, 0))
    with pytest.raises(binding.D3Error) as e:
        binding.Decoder(SMALL_BF16, w, 1, 32, kv_dtype="bf16")
    assert "D3_BF16" in str(e.value)


@pytest.mark.parametrize("B", [1, 2, 3, 4])
def test_tiny_fp32_batches_use_the_alu_path(B):
    _run(d3_inputs.TINY, B, 9, 8, 0.9, 1, kv_dtype="f32", forced_seed=6)


@pytest.mark.parametrize("B,P", [(1, 16), (2, 7), (5, 13), (16, 3), (17, 4), (32, 2)])
def test_small_bf16_matrix_core_path(B, P):
    # B = 1 decodes on the vector ALUs and prefills on the matrix cores; B >= 2 uses the matrix cores throughout
    _run(SMALL_BF16, B, P, 8, 0.9, 2, forced_seed=7)


@pytest.mark.parametrize("shape,B,P", [(SMALL_BF16, 2, 24), (SMALL_BF16, 2, 97), (SMALL_BF16, 1, 81), (SMALL_GQA, 1, 80),
                                       (SMALL_GQA, 2, 72), (SMALL_GQA, 1, 128), (SMALL_BF16, 2, 50), (SMALL_GQA, 1, 168),
                                       (SMALL_GQA, 1, 136), (SMALL_BF16, 1, 144), (SMALL_GQA, 2, 145)])
def test_prompt_lengths_that_end_in_every_chunk_width(shape, B, P):
    # the prompt pass takes one sequence at a time in chunks of up to 1024 columns; the chunks here have 24, 97, 81, 80, 72,
    # 128, 50, 168, 136, 144 and 145 columns, which ends in each of the projection kernels (packed, 16-column, the panel
    # kernel with two, four and eight column tiles, and the LDS-tiled kernel with a ragged second column block) and in both
    # attention paths of a prompt chunk (per column on the vector ALUs at head_dim 64, query tiles on the matrix cores at 128)
    _run(shape, B, P, 4, 0.8, 1, forced_seed=9)


def test_wide_prompt_chunks_as_two_launches_of_64_columns(monkeypatch):
    # what the projections of large matrices (hundreds of MB) do with a chunk of more than 64 columns, forced on small ones
    monkeypatch.setenv("D3_WIDE_SPLIT_MB", "0")
    _run(SMALL_GQA, 2, 150, 4, 0.8, 1, forced_seed=9)
    _run(SMALL_BF16, 1, 97, 4, 0.8, 1, forced_seed=9)


@pytest.mark.parametrize("cols", [64, 128, 256])
def test_prompt_chunks_of_a_forced_width(monkeypatch, cols):
    # a prompt of 700 tokens in chunks of 64 or 128 columns (panel kernel) and of 256 (LDS-tiled kernel: two full chunks
    # and one of 188 columns, whose second column block is ragged)
    monkeypatch.setenv("D3_PREFILL_COLS", str(cols))
    _run(SMALL_GQA, 2, 150 if cols == 64 else 700, 4, 0.8, 1, forced_seed=9)


@pytest.mark.parametrize("ks", [2, 3, 4])
def test_prompt_residual_projections_in_k_parts(monkeypatch, ks):
    # the residual projections of a prompt chunk with K cut into 2, 3 and 4 parts (one workgroup each; the part that arrives
    # last at the tile's counter adds the published accumulators in part order): K of 16 and 43 stages (uneven parts),
    # then 8 and 22 stages; by itself the launcher cuts K only for long contractions (the 7B / 13B / 70B widths, which
    # the all-block and full-size tests run)
    monkeypatch.setenv("D3_PROMPT_KS", str(ks))
    _run(SMALL_GQA, 1, 300, 3, 0.8, 1, forced_seed=21)
    _run(SMALL_BF16, 2, 200, 3, 0.9, 2, forced_seed=21)


def test_lds_tiled_prompt_kernel_shapes():
    # rows that do not fill the last row block (d_ffn 1376 = 10.75 blocks of 128 gate/up pairs, vocab 2000), five and a half
    # column blocks; K of 16 stages (four-wave kernel) and 43 stages (odd: the residual projection cannot pair its stages
    # and takes the four-wave kernel too); then head_dim 64 (vector-ALU attention per column) with 1100 tokens, a chunk of
    # 1024 columns and one of 76, K of 8 and 22 stages (even: the residual projections run the eight-wave kernel, whose
    # steady-state loop runs twice and nine times before its four-stage tail)
    _run(SMALL_GQA, 1, 700, 3, 0.8, 1, forced_seed=19)
    _run(SMALL_BF16, 1, 1100, 3, 0.9, 2, forced_seed=19)
    # the shortest contractions: K of 4 stages (the eight-wave kernel is all prologue and tail) and of 6 (one steady-state turn)
    _run(ModelShape("narrow", L=2, d=128, H=2, H_kv=1, hd=64, F=192, V=512, dtype="bf16"), 1, 300, 3, 0.9, 1, forced_seed=19)


@pytest.mark.parametrize("B,kv", [(1, "f16"), (3, "f16"), (2, "f32")])
def test_small_gqa(B, kv):
    _run(SMALL_GQA, B, 37, 6, 0.8, 1, forced_seed=8, kv_dtype=kv)


@pytest.mark.parametrize("B,P", [(2, 300), (1, 700)])
def test_fp32_cache_on_the_matrix_core_attention_kernels(B, P):
    # grouped-query attention at head_dim 128 with an fp32 cache (what models deeper than 48 blocks get): the cache rows go
    # to the matrix cores as fp16 hi + lo planes; prompt chunks of 128 + 128 + 44 columns (query tiles), decode contexts
    # that span three and six splits, batch 1 (vector-ALU projections) and batch 2 (matrix-core projections).  The fp32
    # rows leave nothing but arithmetic rounding: the logits must agree 100 times closer than the acceptance bound.
    gpu, gens = _run(SMALL_GQA, B, P, 5, 0.8, 1, forced_seed=8, kv_dtype="f32")
    helpers.compare(gpu, gens, 5, logit_atol=2e-4, hidden_tol=1e-4)


@pytest.mark.parametrize("kv", ["f16", "f32"])
def test_batch1_decode_grouped_query_head_dim_128(kv):
    _run(SMALL_GQA, 1, 70, 12, 0.85, 1, forced_seed=14, kv_dtype=kv)


def test_batch1_zero_blocks_and_free_running_tokens():
    gpu, gens = _run(SMALL_GQA, 1, 9, 6, 0.5, 1)      # keep = 3, 1, 0, 0, ...: steps with no block at all
    assert gens[0].keep[2] == 0


def test_long_context_spans_several_attention_splits():
    _run(SMALL_BF16, 2, 700, 4, 0.9, 2, forced_seed=9)


def test_window_at_block_zero_and_min_keep():
    _run(SMALL_BF16, 2, 5, 10, 0.7, 0, forced_seed=10, min_keep=1)


def test_zero_blocks_kept():
    # alpha = 0.5 on 4 blocks: keep = 4, 2, 1, 0, 0: the last steps run the embedding and lm_head only
    _run(SMALL_BF16, 1, 4, 5, 0.5, 1, forced_seed=11)


def test_llama7b_widths_two_blocks_batch1():
    _run(d3_inputs.LLAMA_7B.truncated(2), 1, 8, 5, 0.7, 1, forced_seed=12)


def test_llama7b_widths_two_blocks_batch4():
    _run(d3_inputs.LLAMA_7B.truncated(2), 4, 3, 3, 0.7, 1, forced_seed=13)


def test_llama13b_widths_one_block_batch4():
    # 13B widths, batch 4: the matrix-core path with one column tile at real K (5120 / 13824) and row counts
    _run(d3_inputs.LLAMA_13B.truncated(1), 4, 2, 3, 1.0, 0, forced_seed=15)


def test_llama70b_widths_one_block_gqa():
    # 70B widths: grouped-query attention (64 query / 8 KV heads) and d_ffn 28672, which only the matrix-core
    # path can take (batch 1 included); one set of weights serves both batch sizes
    shape = d3_inputs.LLAMA_70B.truncated(1)
    w = d3_inputs.make_weights(shape, 0)
    for B in (2, 1):
        prompts = d3_inputs.make_prompt(B, 2, shape.V, seed=1)
        forced = _forced(B, 2, shape.V, 16)
        print(f"case {shape.name} B={B}", flush=True)
        gpu = helpers.gpu_generate(shape, w, prompts, 2, 1.0, 0, forced=forced)
        _, gens = helpers.oracle_generate(shape, w, prompts, 2, 1.0, 0, forced=forced)
        wl, wh = helpers.compare(gpu, gens, 2)
        print(f"  worst logit abs err {wl:.3e}, worst hidden rel L2 {wh:.3e}", flush=True)
        del gpu


def test_full_size_7b_configuration_sampled_against_oracle():
    """The benchmark's own launch configuration (7B shape, 32 blocks, batch 1, prompt 512) checked on the
    outputs the oracle can afford: the hidden state after block 0 of the last prompt position and of every
    decode step, and the complete logits of the steps that keep only block 0 / no block (alpha = 0.5 keeps
    32, 16, 8, 4, 2, 1, 0 blocks).  All 32 blocks point at the same weight tensors, so the host draws one
    block; the oracle runs that block alone over the 518 rows."""
    import torch
    from oracle import oracle
    from paper_2503_08524_amd import binding

    full = d3_inputs.LLAMA_7B
    one = full.truncated(1)
    w1 = d3_inputs.make_weights(one, 0)
    w_tied = dict(w1)
    w_tied["layers"] = [w1["layers"][0]] * full.L
    P, G, alpha, start = 512, 7, 0.5, 19
    prompts = d3_inputs.make_prompt(1, P, full.V, seed=1)
    forced = _forced(1, G, full.V, 17)
    keep, drop, ids = binding.d3_plan_depth(full.L, alpha, start, 0, G)
    assert keep.tolist() == [32, 16, 8, 4, 2, 1, 0] and ids[5, 0] == 0

    # GPU: the real thing, one device copy of the block shared by all 32 layer entries
    dev = binding.weights_to_device(one, w1)
    dev_tied = dict(dev)
    dev_tied["layers"] = [dev["layers"][0]] * full.L
    dec = binding.Decoder(full, dev_tied, 1, P + G)
    print("case full-size 7B, tied blocks", flush=True)
    gpu = helpers.gpu_generate(full, None, prompts, G, alpha, start, forced=forced, decoder=dec, fill_each_step=True)

    # oracle: block 0 alone over every row
    oracle.set_threads(helpers.oracle_threads())
    model = oracle.OracleModel(one, w1)
    seq = model.new_seq(P + G)
    hid = None
    for p in range(P):
        hid, _ = seq.forward_token(int(prompts[0, p]), p, [0], want_hidden=(p == P - 1))
    def rel(a, b):
        return float(np.linalg.norm(a - b) / np.linalg.norm(b))
    assert rel(gpu["hidden"][0][1, 0].astype(np.float64), hid[1]) <= helpers.HIDDEN_REL_L2
    worst = 0.0
    for i in range(1, G):
        blocks = [0] if keep[i] >= 1 else []
        h, lg = seq.forward_token(int(forced[0, i - 1]), P + i - 1, blocks, want_hidden=True, want_logits=True)
        got = gpu["hidden"][i][:, 0].astype(np.float64)
        assert rel(got[0], h[0]) <= 1e-6                                   # the embedding row
        if keep[i] >= 1:
            assert rel(got[1], h[1]) <= helpers.HIDDEN_REL_L2, f"step {i}"
        if keep[i] <= 1:                                                    # logits depend on block 0 at most
            err = float(np.abs(gpu["logits"][i][0].astype(np.float64) - lg).max())
            worst = max(worst, err)
            assert err <= helpers.LOGIT_ATOL, f"step {i}: logits max abs err {err:.3e}"
            top2 = np.partition(lg, -2)[-2:]
            if top2[1] - top2[0] > helpers.TOKEN_MARGIN:
                assert int(gpu["tokens"][i][0]) == oracle.argmax(lg)
    print(f"  worst logit abs err {worst:.3e}", flush=True)
    # the fill of the dropped blocks copied the source block's rows (bit-exact), at full cache size
    for i in (1, 5):
        pos, s, n = P + i - 1, int(drop[i]), full.L - int(keep[i])
        src = s - 1
        assert torch.equal(dec.k_cache[s, 0, :, pos], dec.k_cache[src, 0, :, pos])
        assert torch.equal(dec.v_cache[s + n - 1, 0, :, pos], dec.v_cache[src, 0, :, pos])


@pytest.mark.timeout(400)
@pytest.mark.parametrize("name,B,P", [("llama-13b", 4, 1024), ("llama-7b", 32, 2048), ("llama-70b", 8, 1024)])
def test_full_size_batched_configurations_sampled_against_oracle(name, B, P):
    """The batched benchmark configurations in their own launch configuration (all blocks, full batch, full prompt),
    checked on what the oracle can afford for two sampled sequences (the first and the last of the batch): the hidden
    state after block 0 of the last prompt position and of every decode step, and the complete logits of the steps that
    keep only block 0 / no block (alpha = 0.5 halves the depth every step).  All blocks point at the same weight
    tensors, so the host draws one block.  For a sampled sequence the oracle fills block 0's cache rows of the prompt
    with its cache-write-only entry (those rows depend on the embeddings alone) and runs block 0 in full for the rows
    that are compared."""
    import torch
    from oracle import oracle
    from paper_2503_08524_amd import binding

    full = d3_inputs.SHAPES[name]
    one = full.truncated(1)
    w1 = d3_inputs.make_weights(one, 0)
    alpha, start = 0.5, d3_inputs.start_layer_from_fraction(full.L, 0.6)
    G = int(np.floor(np.log2(full.L))) + 2                       # depth L, L/2, ..., 1, 0
    keep, drop, ids = binding.d3_plan_depth(full.L, alpha, start, 0, G)
    assert keep[0] == full.L and keep[G - 2] == 1 and keep[G - 1] == 0 and all(ids[i, 0] == 0 for i in range(G - 1))
    prompts = d3_inputs.make_prompt(B, P, full.V, seed=1)
    forced = _forced(B, G, full.V, 17)

    dev = binding.weights_to_device(one, w1)
    dev_tied = dict(dev)
    dev_tied["layers"] = [dev["layers"][0]] * full.L
    dec = binding.Decoder(full, dev_tied, B, P + G)
    print(f"case full-size {name} B={B} P={P}, tied blocks", flush=True)
    gpu = helpers.gpu_generate(full, None, prompts, G, alpha, start, forced=forced, decoder=dec, fill_each_step=True)

    oracle.set_threads(helpers.oracle_threads())
    model = oracle.OracleModel(one, w1)
    def rel(a, b):
        return float(np.linalg.norm(a - b) / np.linalg.norm(b))
    worst_l = worst_h = 0.0
    for b in (0, B - 1):
        seq = model.new_seq(P + G)
        for p in range(P - 1):
            seq.first_block_kv(int(prompts[b, p]), p, 0)
        hid, _ = seq.forward_token(int(prompts[b, P - 1]), P - 1, [0], want_hidden=True)
        e = rel(gpu["hidden"][0][1, b].astype(np.float64), hid[1])
        worst_h = max(worst_h, e)
        assert e <= helpers.HIDDEN_REL_L2, f"seq {b} prompt: hidden rel L2 {e:.3e}"
        for i in range(1, G):
            blocks = [0] if keep[i] >= 1 else []
            h, lg = seq.forward_token(int(forced[b, i - 1]), P + i - 1, blocks, want_hidden=True, want_logits=True)
            got = gpu["hidden"][i][:, b].astype(np.float64)
            assert rel(got[0], h[0]) <= 1e-6                               # the embedding row
            if keep[i] >= 1:
                e = rel(got[1], h[1])
                worst_h = max(worst_h, e)
                assert e <= helpers.HIDDEN_REL_L2, f"seq {b} step {i}: hidden rel L2 {e:.3e}"
            if keep[i] <= 1:                                                # logits depend on block 0 at most
                err = float(np.abs(gpu["logits"][i][b].astype(np.float64) - lg).max())
                worst_l = max(worst_l, err)
                assert err <= helpers.LOGIT_ATOL, f"seq {b} step {i}: logits max abs err {err:.3e}"
                top2 = np.partition(lg, -2)[-2:]
                if top2[1] - top2[0] > helpers.TOKEN_MARGIN:
                    assert int(gpu["tokens"][i][b]) == oracle.argmax(lg)
    print(f"  worst logit abs err {worst_l:.3e}, worst hidden rel L2 {worst_h:.3e}", flush=True)
    # the fill of the dropped blocks copied the source block's rows (bit-exact), at full cache size
    i = 1
    pos, s, n = P + i - 1, int(drop[i]), full.L - int(keep[i])
    assert s >= 1 and torch.equal(dec.k_cache[s, B - 1, :, pos], dec.k_cache[s - 1, B - 1, :, pos])
    assert torch.equal(dec.v_cache[s + n - 1, 0, :, pos], dec.v_cache[s - 1, 0, :, pos])
    dec.close()
