"""The byte accounting behind the reported HBM fractions (no GPU): bench.algorithmic_bytes against totals worked out by
hand from the shapes (weights of the kept blocks + KV rows read and appended + fill + lm_head, per decode step)."""
import numpy as np
import pytest

import bench
import d3_inputs
from oracle import oracle

# (config, alpha, GB per decode step averaged over the request), fp16/bf16 cache, COPY fill
EXPECTED = [("7b", 1.0, 13.550), ("7b", 0.995, 7.529), ("7b", 0.99, 4.800),
            ("13b", 1.0, 29.481), ("13b", 0.995, 16.336),
            ("7b-b32", 1.0, 51.886), ("7b-b32", 0.995, 17.422),
            ("70b", 1.0, 140.449), ("70b", 0.995, 78.393)]


@pytest.mark.parametrize("cfg,alpha,gb", EXPECTED)
def test_algorithmic_bytes_per_step(cfg, alpha, gb):
    shape, B, P, G, _, start_frac = bench.CONFIGS[cfg]
    start = d3_inputs.start_layer_from_fraction(shape.L, start_frac)
    keep, _, _ = oracle.plan_depth(shape.L, alpha, start, 0, G)
    total = bench.algorithmic_bytes(shape, B, P, G, keep, 2, "copy")
    assert total / (G - 1) / 1e9 == pytest.approx(gb, rel=2e-3)


def test_block_weight_bytes_of_the_7b_shape():
    s = d3_inputs.LLAMA_7B
    # 4 d^2 (q, k, v, o) + 3 d F (gate, up, down) parameters, two bytes each; the norm gains are not counted
    assert bench.block_weight_bytes(s) == 2 * (4 * 4096 * 4096 + 3 * 4096 * 11008)


def test_ragged_batch_counts_its_own_rows():
    s = d3_inputs.LLAMA_7B
    keep = np.full(8, s.L)
    full = bench.algorithmic_bytes(s, 4, 512, 8, keep, 2, "none")
    ragged = bench.algorithmic_bytes(s, 4, 512, 8, keep, 2, "none", prompt_rows=512 + 384 + 256 + 128)
    kv_row = 2 * s.H_kv * s.hd * 2
    assert full - ragged == 7 * s.L * kv_row * (4 * 512 - 1280)
