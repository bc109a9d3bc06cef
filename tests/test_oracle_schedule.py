"""Pins of the oracle's depth schedule (no GPU): closed form vs exact rationals,
the averages the paper prints, structural invariants, FLOPs-reduction column."""
import os
from fractions import Fraction

import numpy as np
import pytest

import d3_inputs
from oracle import bruteforce, oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# (L, alpha) of the benchmark configurations and of the paper's grids (Table 4, Section 4.1)
GRID = [(L, a) for L in (4, 32, 40, 80) for a in ("1.0", "0.97", "0.995", "0.99", "0.8", "0.9", "0.999", "0.9999")]


@pytest.mark.parametrize("L,alpha", GRID)
def test_keep_matches_exact_rational(L, alpha):
    n = 1231  # longest GSM8K output in Table 3 is 1230 tokens
    keep, _, _ = oracle.plan_depth(L, float(alpha), 0, 0, n)
    p = Fraction(1)
    a = Fraction(alpha)
    for i in range(n):
        v = L * p
        assert keep[i] == v.numerator // v.denominator, (L, alpha, i)
        p *= a


def test_keep_matches_libm_pow_at_configs():
    for L, alpha in [(4, 0.97), (32, 0.995), (32, 0.99), (40, 0.995), (80, 0.995)]:
        keep, _, _ = oracle.plan_depth(L, alpha, 1, 0, 512)
        assert [int(np.floor(L * alpha ** i)) for i in range(512)] == keep.tolist()


def test_tiny_config_keep_run_lengths():
    # L=4, alpha=0.97, 32 tokens: 4 once, then 3, 2, 1 (checked by hand: 4*0.97 = 3.88,
    # 4*0.97^10 = 2.95, 4*0.97^23 = 1.99)
    keep, _, _ = oracle.plan_depth(4, 0.97, 2, 0, 32)
    assert keep.tolist() == [4] + [3] * 9 + [2] * 13 + [1] * 9


@pytest.mark.parametrize("L,alpha,maxlen,printed", _rows("table5_gsm8k_avg_layers.txt"))
def test_table5_average_layers(L, alpha, maxlen, printed):
    L, maxlen = int(L), int(maxlen)
    for start in (d3_inputs.start_layer_from_fraction(L, f) for f in (0.2, 0.6, 0.8)):
        keep, _, _ = oracle.plan_depth(L, float(alpha), start, 0, maxlen + 1)
        # the printed two decimals do not depend on whether i starts at 0 or 1, nor on `start`
        assert f"{keep[:maxlen].mean():.2f}" == printed
        assert f"{keep[1:maxlen + 1].mean():.2f}" == printed


@pytest.mark.parametrize("L", [4, 32, 40, 80])
@pytest.mark.parametrize("alpha", [1.0, 0.9999, 0.995, 0.99, 0.9, 0.8])
def test_structural_invariants(L, alpha):
    n = 400
    for start in sorted({0, 1, L // 2, d3_inputs.start_layer_from_fraction(L, 0.6), L - 1}):
        keep, drop, ids = oracle.plan_depth(L, alpha, start, 0, n)
        assert keep[0] == L
        assert (np.diff(keep) <= 0).all()
        prev = set()
        for i in range(n):
            executed = [int(x) for x in ids[i] if x >= 0]
            assert len(executed) == keep[i] and executed == sorted(set(executed))
            assert (ids[i, keep[i]:] == -1).all()
            dropped = sorted(set(range(L)) - set(executed))
            assert dropped == list(range(drop[i], drop[i] + L - keep[i]))      # contiguous window
            if dropped and start + len(dropped) <= L:
                assert dropped[0] == start                                     # window starts at `start` while it fits
            assert prev <= set(dropped)                                        # nested: never un-skip a block
            prev = set(dropped)
            assert executed == bruteforce.executed_blocks(L, repr(alpha), start, i)
        if alpha == 1.0:
            assert (keep == L).all()


def test_min_keep_and_zero_blocks():
    keep, drop, ids = oracle.plan_depth(32, 0.8, 19, 0, 40)
    assert keep[16] == 0 and keep[15] == 1 and (ids[16] == -1).all()
    keep2, _, _ = oracle.plan_depth(32, 0.8, 19, 3, 40)
    assert keep2.min() == 3 and (keep2 == np.maximum(keep, 3)).all()


def test_plan_rejects_bad_arguments():
    for args in [(0, 0.9, 0, 0, 4), (4, 0.0, 0, 0, 4), (4, 1.5, 0, 0, 4), (4, 0.9, 4, 0, 4), (4, 0.9, -1, 0, 4),
                 (4, float("nan"), 0, 0, 4), (4, 0.9, 0, 5, 4)]:
        with pytest.raises(ValueError):
            oracle.plan_depth(*args)


@pytest.mark.parametrize("model,L,avg,printed", _rows("table5_flops_reduction.txt"))
def test_table5_flops_reduction(model, L, avg, printed):
    s = d3_inputs.SHAPES[model]
    r = oracle.flops_reduction(int(L), float(avg), s.d, s.V, s.params_per_block)
    assert abs(r - float(printed)) <= 0.0101, (model, avg, r, printed)


# ---------- linear decay between bounds (the comparison schedule of Section 3.4 / Section 4.1) ----------

@pytest.mark.parametrize("L,first,last,n", [(32, 32, 8, 256), (32, 32, 17, 200), (40, 36, 4, 1024), (80, 80, 0, 77), (4, 4, 1, 32),
                                           (32, 20, 20, 9), (32, 32, 31, 2), (8, 8, 2, 1)])
def test_linear_keep_matches_exact_rational_line_and_its_invariants(L, first, last, n):
    keep, drop, ids = oracle.plan_depth_linear(L, first, last, L // 2, n)
    assert keep.tolist() == [bruteforce.kept_blocks_linear(L, first, last, n, i) for i in range(n)]
    assert keep[0] == first and (n == 1 or keep[-1] == last)              # the bounds are reached
    assert (np.diff(keep) <= 0).all()                                     # never deeper later
    if n > 1:                                                             # never more than one line-step below the line
        line = first - (first - last) * np.arange(n) / (n - 1)
        assert ((line - keep >= 0) & (line - keep < 1)).all()
    for i in range(n):
        assert ids[i, : keep[i]].tolist() == bruteforce.executed_blocks_linear(L, first, last, n, L // 2, i)
        assert (ids[i, keep[i]:] == -1).all()


def test_linear_is_an_arithmetic_progression_when_the_step_divides():
    # 32 -> 8 over 25 steps loses exactly one block per step; over 49 steps one block every other step
    keep, _, _ = oracle.plan_depth_linear(32, 32, 8, 0, 25)
    assert keep.tolist() == list(range(32, 7, -1))
    keep, _, _ = oracle.plan_depth_linear(32, 32, 8, 0, 49)
    assert keep[::2].tolist() == list(range(32, 7, -1)) and (keep[1::2] == keep[2::2]).all()
    assert keep.sum() * 2 == (32 + 8) * 49 - 24                             # mean of the line minus the 24 half-steps floored away


def test_linear_directions_head_first_and_tail_first():
    L, n = 12, 23
    keep, drop, ids = oracle.plan_depth_linear(L, 12, 1, 0, n)            # shallow blocks go first
    for i in range(n):
        assert ids[i, : keep[i]].tolist() == list(range(L - keep[i], L))
    keep, drop, ids = oracle.plan_depth_linear(L, 12, 1, L - 1, n)        # deep blocks go first: an early exit
    for i in range(n):
        assert ids[i, : keep[i]].tolist() == list(range(keep[i]))


def test_linear_plan_rejects_bad_arguments():
    for args in [(0, 0, 0, 0, 4), (8, 9, 2, 0, 4), (8, 4, 5, 0, 4), (8, 8, -1, 0, 4), (8, 8, 2, 8, 4), (8, 8, 2, -1, 4), (8, 8, 2, 0, -1)]:
        with pytest.raises(ValueError):
            oracle.plan_depth_linear(*args)
