"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol the header
declares, and the host-only schedule entry point agrees with the oracle bit for bit."""
import os
import re

import numpy as np
import pytest

import d3_inputs
import paper_2503_08524_amd as d3
from oracle import oracle
from paper_2503_08524_amd import build as d3_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if d3_build.is_stale():
        d3_build.build()
    return d3.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "d3.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(d3_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"d3_plan_depth", "d3_prefill", "d3_decode_step", "d3_fill_missing_kv", "d3_create", "d3_destroy",
            "d3_set_plan", "d3_workspace_size", "d3_last_error", "d3_n_ctx"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


@pytest.mark.parametrize("L,alpha,start", [(4, 0.97, 2), (32, 0.995, 19), (32, 0.99, 19), (40, 0.995, 24), (80, 0.995, 48),
                                           (32, 1.0, 19), (32, 0.8, 0), (80, 0.9999, 16), (40, 0.9, 39)])
def test_plan_is_bit_exact_against_oracle(lib, L, alpha, start):
    for min_keep in (0, 2):
        got = d3.d3_plan_depth(L, alpha, start, min_keep, 1300)
        ref = oracle.plan_depth(L, alpha, start, min_keep, 1300)
        for g, r in zip(got, ref):
            assert (g == r).all()


@pytest.mark.parametrize("L,first,last,start", [(32, 32, 8, 0), (32, 32, 17, 31), (40, 36, 4, 24), (80, 80, 0, 48), (4, 4, 1, 2), (32, 20, 20, 5)])
def test_linear_plan_is_bit_exact_against_oracle_and_survives_the_table_entry(lib, L, first, last, start):
    for n in (1, 2, 77, 1024):
        got = d3.d3_plan_depth_linear(L, first, last, start, n)
        ref = oracle.plan_depth_linear(L, first, last, start, n)
        for g, r in zip(got, ref):
            assert (g == r).all()
        assert (d3.d3_plan_from_table(L, ref[0], ref[1]) == ref[2]).all()


def test_plan_table_rejects_steps_that_do_not_fit(lib):
    for keep, drop in [([5], [0]), ([-1], [0]), ([2], [3]), ([2], [-1]), ([4, 3, 1], [0, 0, 2])]:
        with pytest.raises(d3.D3Error) as e:
            d3.d3_plan_from_table(4, keep, drop)
        assert e.value.status == -1 and "d3_plan_from_table" in str(e.value)
    assert d3.d3_plan_from_table(4, [4, 3, 0], [4, 3, 0]).tolist() == [[0, 1, 2, 3], [0, 1, 2, -1], [-1, -1, -1, -1]]
    with pytest.raises(d3.D3Error):
        d3.d3_plan_depth_linear(8, 9, 2, 0, 4)


def test_plan_from_table_lists_exactly_the_blocks_outside_each_window(lib):
    rng = np.random.default_rng(7)
    for _ in range(200):
        L = int(rng.integers(1, 90))
        n = int(rng.integers(1, 40))
        keep = rng.integers(0, L + 1, size=n)
        drop = np.array([int(rng.integers(0, k + 1)) for k in keep])       # window [drop, drop + L - keep) ends at or before L
        ids = d3.d3_plan_from_table(L, keep, drop)
        for i in range(n):
            want = [l for l in range(L) if not (drop[i] <= l < drop[i] + L - keep[i])]
            assert ids[i, : keep[i]].tolist() == want and (ids[i, keep[i]:] == -1).all()


def test_plan_accepts_null_outputs_and_zero_steps(lib):
    assert lib.d3_plan_depth(8, 0.9, 3, 0, 5, None, None, None) == 0
    assert lib.d3_plan_depth(8, 0.9, 3, 0, 0, None, None, None) == 0


@pytest.mark.parametrize("args", [(0, 0.9, 0, 0, 4), (4, 0.0, 0, 0, 4), (4, 1.0001, 0, 0, 4), (4, float("nan"), 0, 0, 4),
                                  (4, 0.9, 4, 0, 4), (4, 0.9, -1, 0, 4), (4, 0.9, 0, 5, 4), (4, 0.9, 0, -1, 4), (4, 0.9, 0, 0, -1)])
def test_plan_rejects_bad_arguments(lib, args):
    with pytest.raises(d3.D3Error) as e:
        d3.d3_plan_depth(*args)
    assert e.value.status == -1 and "d3_plan_depth" in str(e.value)


def test_workspace_size_and_shape_checks(lib):
    for s in (d3_inputs.TINY, d3_inputs.LLAMA_7B, d3_inputs.LLAMA_13B, d3_inputs.LLAMA_70B):
        n = d3.d3_workspace_size(s, "f16" if s.dtype == "bf16" else "f32", 8, 2048)
        assert n > 0 and n % 256 == 0 and n < 2 ** 31
    bad = d3_inputs.ModelShape("bad", L=2, d=256, H=4, H_kv=3, hd=64, F=688, V=1024)
    assert d3.d3_workspace_size(bad, "f16", 1, 64) == 0
    assert "n_kv_heads" in lib.d3_last_error().decode()
    bad = d3_inputs.ModelShape("bad", L=2, d=256, H=4, H_kv=4, hd=80, F=688, V=1024)
    assert d3.d3_workspace_size(bad, "f16", 1, 64) == 0
    assert d3.d3_workspace_size(d3_inputs.TINY, "f32", 33, 64) == 0          # max_batch beyond 32
    assert d3.d3_workspace_size(d3_inputs.LLAMA_7B, "bf16", 1, 64) == 0       # a bf16 cache misses the logit tolerance
    assert "D3_BF16" in lib.d3_last_error().decode()


def test_null_context_is_an_error_not_a_crash(lib):
    assert lib.d3_set_plan(None, 0.9, 0, 0, 4) == -1
    assert lib.d3_decode_step(None, None, 1, None, None, None, None) == -1
    assert lib.d3_prefill(None, None, 1, 1, 0, None, None, None, None) == -1
    assert lib.d3_fill_missing_kv(None, 0, 0, 0, None) == -1
    assert lib.d3_n_ctx(None) == 0
    assert lib.d3_destroy(None) == 0
