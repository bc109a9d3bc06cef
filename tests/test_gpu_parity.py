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
    _, gens = helpers.oracle_generate(shape, w, prompts, G, alpha, start, forced=forced, min_keep=kw.get("min_keep", 0))
    wl, wh = helpers.compare(gpu, gens, G, check_tokens=check_tokens)
    print(f"  worst logit abs err {wl:.3e}, worst hidden rel L2 {wh:.3e}", flush=True)
    return gpu, gens


@pytest.mark.parametrize("alpha", [0.97, 1.0])
def test_tiny_config_tokens_logits_hidden(alpha):
    # the first benchmark configuration in full: fp32 weights, fp32 cache, free-running greedy decoding
    gpu, gens = _run(d3_inputs.TINY, 1, 16, 32, alpha, 2, kv_dtype="f32", check_tokens="all")
    helpers.compare(gpu, gens, 32, check_tokens="all", logit_atol=1e-4, hidden_tol=1e-5)


def test_tiny_config_bf16_cache():
    _run(d3_inputs.TINY, 1, 16, 32, 0.97, 2, kv_dtype="bf16", forced_seed=5)


@pytest.mark.parametrize("B", [1, 2, 3, 4])
def test_tiny_fp32_batches_use_the_alu_path(B):
    _run(d3_inputs.TINY, B, 9, 8, 0.9, 1, kv_dtype="f32", forced_seed=6)


@pytest.mark.parametrize("B,P", [(1, 16), (2, 7), (5, 13), (16, 3), (17, 4), (32, 2)])
def test_small_bf16_matrix_core_path(B, P):
    # B = 1 decodes on the vector ALUs and prefills on the matrix cores; B >= 2 uses the matrix cores throughout
    _run(SMALL_BF16, B, P, 8, 0.9, 2, forced_seed=7)


@pytest.mark.parametrize("B,kv", [(1, "f16"), (3, "f16"), (2, "bf16"), (2, "f32")])
def test_small_gqa(B, kv):
    _run(SMALL_GQA, B, 37, 6, 0.8, 1, forced_seed=8, kv_dtype=kv)


@pytest.mark.parametrize("persistent", [True, False])
@pytest.mark.parametrize("kv", ["f16", "bf16", "f32"])
def test_batch1_decode_as_one_persistent_launch_and_as_separate_launches(persistent, kv):
    # head_dim 128, bf16 weights, batch 1: the whole step is one cooperative launch unless switched off
    _run(SMALL_GQA, 1, 70, 12, 0.85, 1, forced_seed=14, kv_dtype=kv, persistent=persistent)


def test_persistent_step_with_zero_blocks_and_free_running_tokens():
    gpu, gens = _run(SMALL_GQA, 1, 9, 6, 0.5, 1, persistent=True)      # keep = 3, 1, 0, 0, ...: steps with no block at all
    assert gens[0].keep[2] == 0


def test_long_context_spans_several_attention_splits():
    _run(SMALL_BF16, 2, 700, 4, 0.9, 2, forced_seed=9)


def test_window_at_block_zero_and_min_keep():
    _run(SMALL_BF16, 2, 5, 10, 0.7, 0, forced_seed=10, min_keep=1)


def test_zero_blocks_kept():
    # alpha = 0.5 on 4 blocks: keep = 4, 2, 1, 0, 0: the last steps run the embedding and lm_head only
    _run(SMALL_BF16, 1, 4, 5, 0.5, 1, forced_seed=11)


@pytest.mark.parametrize("persistent", [True, False])
def test_llama7b_widths_two_blocks_batch1(persistent):
    _run(d3_inputs.LLAMA_7B.truncated(2), 1, 8, 5, 0.7, 1, forced_seed=12, persistent=persistent)


def test_llama7b_widths_two_blocks_batch4():
    _run(d3_inputs.LLAMA_7B.truncated(2), 4, 3, 3, 0.7, 1, forced_seed=13)
