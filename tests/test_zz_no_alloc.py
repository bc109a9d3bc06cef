"""d3_decode_step_static (the decode step for callers that cannot allocate: its intermediates live in a static device
array inside the library) against d3_decode_step, through the C ABI: two requests in a row on the same GPU, the second
a smaller model at a smaller batch, so the array still holds the first one's contents, in another layout, when the
second one runs.  Same kernels, same launch shapes, same summation orders: every output must be identical."""
import numpy as np
import pytest

import d3_inputs
from d3_inputs import ModelShape

pytestmark = pytest.mark.gpu

BIG = ModelShape("static-gqa", L=3, d=512, H=8, H_kv=2, hd=128, F=1376, V=2000, dtype="bf16")
SMALL = ModelShape("static-mha", L=4, d=256, H=4, H_kv=4, hd=64, F=704, V=1024, dtype="bf16")


def _request(shape, B, P, G, static, lengths=None, kv=None):
    """Prompt pass + G-1 decode steps (teacher-forced), each through d3_decode_step or d3_decode_step_static."""
    import torch
    from paper_2503_08524_amd import binding
    dev = "cuda:0"
    w = binding.weights_to_device(shape, d3_inputs.make_weights(shape, 3), dev)
    dec = binding.Decoder(shape, w, B, P + G, kv_dtype=kv, device=dev)
    keep, _, _ = binding.d3_plan_depth(shape.L, 0.8, 1, 0, G)
    dec.set_plan(0.8, 1, 0, G)
    prompts = torch.from_numpy(d3_inputs.make_prompt(B, P, shape.V, seed=5)).to(dev)
    forced = torch.from_numpy(d3_inputs.make_prompt(B, G, shape.V, seed=6)).to(dev)
    if lengths is None:
        dec.prefill(prompts)
    else:
        dec.prefill_ragged(prompts, lengths)
    ws_before = dec.workspace.clone()
    out = []
    nxt = torch.zeros(B, dtype=torch.int32, device=dev)
    logits = torch.zeros(B, shape.V, dtype=torch.float32, device=dev)
    for i in range(1, G):
        hid = torch.zeros(int(keep[i]) + 1, B, shape.d, dtype=torch.float32, device=dev)
        step = dec.decode_step_static if static else dec.decode_step
        step(forced[:, i].contiguous(), i, nxt, logits=logits, hidden_dump=hid)
        dec.fill_missing_kv(dec.n_ctx - 1, dec.n_ctx)
        out.append((nxt.cpu().numpy().copy(), logits.cpu().numpy().copy(), hid.cpu().numpy().copy()))
    dec.synchronize()
    if static:      # the context's own workspace was not used
        assert torch.equal(ws_before, dec.workspace)
    cache = (dec.k_cache.cpu().numpy().copy(), dec.v_cache.cpu().numpy().copy())
    dec.close()
    return out, cache


def _same(a, b):
    (out_a, cache_a), (out_b, cache_b) = a, b
    assert len(out_a) == len(out_b)
    for i, ((ta, la, ha), (tb, lb, hb)) in enumerate(zip(out_a, out_b)):
        assert np.array_equal(ta, tb), f"tokens differ at decode step {i + 1}"
        assert np.array_equal(la, lb), f"logits differ at decode step {i + 1}: max abs {np.abs(la - lb).max():.3e}"
        assert np.array_equal(ha, hb), f"hidden states differ at decode step {i + 1}"
    assert np.array_equal(cache_a[0], cache_b[0]) and np.array_equal(cache_a[1], cache_b[1])


def test_static_scratch_step_equals_the_workspace_step_on_two_requests_in_a_row():
    from paper_2503_08524_amd import binding
    assert binding.load_library().d3_static_scratch_bytes() == 32 << 20
    print("case static scratch: batch 5, grouped-query, head_dim 128 (matrix-core path)", flush=True)
    first = _request(BIG, 5, 70, 6, static=True)
    print("case static scratch: batch 1, head_dim 64 (vector-ALU path)", flush=True)
    second = _request(SMALL, 1, 9, 7, static=True)
    print("case static scratch: ragged batch 3", flush=True)
    third = _request(SMALL, 3, 20, 5, static=True, lengths=np.array([20, 4, 11], np.int32))
    _same(first, _request(BIG, 5, 70, 6, static=False))
    _same(second, _request(SMALL, 1, 9, 7, static=False))
    _same(third, _request(SMALL, 3, 20, 5, static=False, lengths=np.array([20, 4, 11], np.int32)))


def test_static_scratch_step_refuses_what_does_not_fit_and_the_recompute_fill():
    import torch
    from paper_2503_08524_amd import binding
    dev = "cuda:0"
    shape = d3_inputs.LLAMA_7B.truncated(1)
    w = binding.random_weights_on_device(shape, 0, dev)
    dec = binding.Decoder(shape, w, 32, 8, device=dev)           # batch 32 at the 7B widths: 40 MB of step buffers
    dec.set_plan(1.0, 0, 0, 4)
    toks = torch.zeros(32, 2, dtype=torch.int32, device=dev)
    cur = dec.prefill(toks)
    nxt = torch.zeros_like(cur)
    with pytest.raises(binding.D3Error) as e:
        dec.decode_step_static(cur, 1, nxt)
    assert e.value.status == -2 and "static array holds" in str(e.value)
    dec.decode_step(cur, 1, nxt)                                 # the refused call changed no state
    dec.close()
    dec = binding.Decoder(SMALL, binding.weights_to_device(SMALL, d3_inputs.make_weights(SMALL, 3), dev), 1, 8, device=dev)
    dec.set_plan(0.8, 1, 0, 4)
    dec.set_fill_mode(binding.D3_FILL_RECOMPUTE)
    cur = dec.prefill(torch.zeros(1, 2, dtype=torch.int32, device=dev))
    with pytest.raises(binding.D3Error) as e:
        dec.decode_step_static(cur, 1, torch.zeros_like(cur))
    assert e.value.status == -4
    dec.close()
