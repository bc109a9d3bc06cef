"""ctypes binding of libd3.so: the same entry points as include/d3.h, argument
marshalling only.  PyTorch supplies device memory and streams; every step of the
path runs in the library's kernels.  There is no fallback: if the library is not
built, loading fails."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None

D3_F32, D3_BF16, D3_F16 = 0, 1, 2
D3_FILL_COPY = 0
D3_FILL_RECOMPUTE = 1
D3_K_NONE, D3_K_QKV, D3_K_ATTN, D3_K_OPROJ, D3_K_GATE_UP, D3_K_DOWN, D3_K_LM_HEAD, D3_K_EMPTY = range(8)


class D3Error(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"d3 status {status}: {message}")
        self.status = status


class _ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_base", C.c_float)] + [
        (n, C.c_int32) for n in ("weight_dtype", "kv_dtype", "max_batch", "max_seq")]


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")]


class _Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("layers", C.POINTER(_LayerWeights)), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


def library_path() -> str:
    return os.environ.get("D3_LIBRARY", os.path.join(_HERE, "libd3.so"))


def load_library() -> C.CDLL:
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise OSError(f"{path} is not built: run `python -m paper_2503_08524_amd.build` (there is no fallback path)")
        # PyTorch ships its own HIP runtime and owns the device memory and streams handed to the library, so it is
        # loaded first: libd3.so then binds to that runtime.  Loaded the other way round the process holds two
        # runtimes and the second one to initialise finds no device.
        import torch  # noqa: F401
        lib = C.CDLL(path)
        i32, vp, dbl = C.c_int32, C.c_void_p, C.c_double
        lib.d3_last_error.restype = C.c_char_p
        lib.d3_plan_depth.argtypes = [i32, dbl, i32, i32, i32, vp, vp, vp]
        lib.d3_plan_depth_linear.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp]
        lib.d3_plan_from_table.argtypes = [i32, i32, vp, vp, vp]
        lib.d3_workspace_size.argtypes = [C.POINTER(_ModelDesc)]
        lib.d3_workspace_size.restype = C.c_size_t
        lib.d3_create.argtypes = [C.POINTER(vp), C.POINTER(_ModelDesc), C.POINTER(_Weights), vp, vp, vp, C.c_size_t]
        lib.d3_destroy.argtypes = [vp]
        lib.d3_set_plan.argtypes = [vp, dbl, i32, i32, i32]
        lib.d3_set_plan_table.argtypes = [vp, vp, vp, i32]
        lib.d3_prefill.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp]
        lib.d3_prefill_ragged.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, vp]
        lib.d3_decode_step.argtypes = [vp, vp, i32, vp, vp, vp, vp]
        lib.d3_decode_step_static.argtypes = [vp, vp, i32, vp, vp, vp, vp]
        lib.d3_static_scratch_bytes.restype = C.c_size_t
        lib.d3_fill_missing_kv.argtypes = [vp, i32, i32, i32, vp]
        lib.d3_set_fill_mode.argtypes = [vp, i32]
        lib.d3_n_ctx.argtypes = [vp]
        lib.d3_n_ctx.restype = i32
        lib.d3_truncate.argtypes = [vp, i32]
        lib.d3_stream_read.argtypes = [vp, vp, C.c_size_t, vp]
        lib.d3_mfma_yardstick.argtypes = [vp, i32, i32, vp]
        lib.d3_profile_select.argtypes = [vp, i32]
        lib.d3_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        _LIB = lib
    return _LIB


def _check(rc: int) -> None:
    if rc != 0:
        raise D3Error(rc, load_library().d3_last_error().decode())


def d3_plan_depth(L: int, alpha: float, start_layer: int, min_keep: int, n_steps: int):
    """(keep[n_steps], drop_begin[n_steps], layer_ids[n_steps][L]) int32 arrays (host only)."""
    keep = np.zeros(max(n_steps, 0), np.int32)
    drop = np.zeros(max(n_steps, 0), np.int32)
    ids = np.zeros((max(n_steps, 0), max(L, 0)), np.int32)
    _check(load_library().d3_plan_depth(L, float(alpha), start_layer, min_keep, n_steps,
                                        keep.ctypes.data, drop.ctypes.data, ids.ctypes.data))
    return keep, drop, ids


def d3_plan_depth_linear(L: int, keep_first: int, keep_last: int, start_layer: int, n_steps: int):
    """Linear decay from keep_first to keep_last; same three arrays as d3_plan_depth (host only)."""
    keep = np.zeros(max(n_steps, 0), np.int32)
    drop = np.zeros(max(n_steps, 0), np.int32)
    ids = np.zeros((max(n_steps, 0), max(L, 0)), np.int32)
    _check(load_library().d3_plan_depth_linear(L, keep_first, keep_last, start_layer, n_steps,
                                               keep.ctypes.data, drop.ctypes.data, ids.ctypes.data))
    return keep, drop, ids


def d3_plan_from_table(L: int, keep, drop_begin):
    """layer_ids[n_steps][L] of a caller-made schedule (host only); raises D3Error on a step that does not fit."""
    keep = np.ascontiguousarray(keep, np.int32); drop = np.ascontiguousarray(drop_begin, np.int32)
    if keep.shape != drop.shape or keep.ndim != 1:
        raise ValueError("keep and drop_begin must be 1-d arrays of one length")
    ids = np.zeros((keep.size, max(L, 0)), np.int32)
    _check(load_library().d3_plan_from_table(L, keep.size, keep.ctypes.data, drop.ctypes.data, ids.ctypes.data))
    return ids


def _desc(shape, kv_dtype: str, max_batch: int, max_seq: int) -> _ModelDesc:
    dt = {"f32": D3_F32, "bf16": D3_BF16, "f16": D3_F16}
    return _ModelDesc(shape.L, shape.d, shape.H, shape.H_kv, shape.hd, shape.F, shape.V, float(shape.eps),
                      float(shape.rope_base), dt[shape.dtype], dt[kv_dtype], max_batch, max_seq)


def d3_workspace_size(shape, kv_dtype: str, max_batch: int, max_seq: int) -> int:
    d = _desc(shape, kv_dtype, max_batch, max_seq)
    return int(load_library().d3_workspace_size(C.byref(d)))


def default_kv_dtype(shape) -> str:
    """Cache precision that keeps logits within 2e-2 of full precision at the model's depth: the rounding of the cache
    rows moves the hidden state by about 4.5e-4 (relative) per block with fp16 rows and grows like sqrt(L), which is
    inside the bound for the 32 and 40 blocks of the 7B and 13B shapes and outside it for the 80 blocks of the 70B shape
    (measured 1.1e-2, 1.7e-2 and 3.3e-2); fp32 rows stay at 4e-4 of logit error at 80 blocks."""
    if shape.dtype == "f32" or shape.L > 48:
        return "f32"
    return "f16"


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Decoder:
    """One d3_ctx plus the device buffers it borrows (all torch tensors on one GPU).

    weights: dict like d3_inputs.make_weights but of torch CUDA tensors
    (float32, or bfloat16 for bf16 models; gains float32).  kv_dtype: "f32" or "f16"; default: default_kv_dtype(shape)."""

    def __init__(self, shape, weights: Dict[str, object], max_batch: int, max_seq: int, kv_dtype: Optional[str] = None,
                 device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.shape = shape
        self.device = torch.device(device)
        self.kv_dtype = kv_dtype or default_kv_dtype(shape)
        self.max_batch, self.max_seq = max_batch, max_seq
        self.weights = weights                       # keep the tensors alive
        desc = _desc(shape, self.kv_dtype, max_batch, max_seq)
        ws_bytes = int(self.lib.d3_workspace_size(C.byref(desc)))
        if ws_bytes == 0:
            _check(-2)
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.kv_dtype]
        kv_shape = (shape.L, max_batch, shape.H_kv, max_seq, shape.hd)
        with torch.cuda.device(self.device):
            self.k_cache = torch.zeros(kv_shape, dtype=tdt, device=self.device)
            self.v_cache = torch.zeros(kv_shape, dtype=tdt, device=self.device)
            self.workspace = torch.zeros(ws_bytes, dtype=torch.uint8, device=self.device)
            layers = (_LayerWeights * shape.L)()
            for l, lw in enumerate(weights["layers"]):
                for name, _ in _LayerWeights._fields_:
                    t = lw[name]
                    assert t.is_cuda and t.is_contiguous(), name
                    setattr(layers[l], name, t.data_ptr())
            self._layers = layers
            w = _Weights(weights["tok_emb"].data_ptr(), layers, weights["final_norm"].data_ptr(), weights["lm_head"].data_ptr())
            ctx = C.c_void_p()
            _check(self.lib.d3_create(C.byref(ctx), C.byref(desc), C.byref(w), self.k_cache.data_ptr(), self.v_cache.data_ptr(),
                                      self.workspace.data_ptr(), ws_bytes))
        self.ctx = ctx

    def close(self) -> None:
        if getattr(self, "ctx", None):
            self.lib.d3_destroy(self.ctx)
            self.ctx = None

    __del__ = close

    def _stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def set_plan(self, alpha: float, start_layer: int, min_keep: int, n_steps: int) -> None:
        _check(self.lib.d3_set_plan(self.ctx, float(alpha), start_layer, min_keep, n_steps))

    def set_plan_table(self, keep, drop_begin) -> None:
        keep = np.ascontiguousarray(keep, np.int32); drop = np.ascontiguousarray(drop_begin, np.int32)
        if keep.shape != drop.shape or keep.ndim != 1:
            raise ValueError("keep and drop_begin must be 1-d arrays of one length")
        _check(self.lib.d3_set_plan_table(self.ctx, keep.ctypes.data, drop.ctypes.data, keep.size))

    def prefill(self, tokens, pos_begin: int = 0, next_tok=None, logits=None, hidden_dump=None):
        """tokens: int32 CUDA tensor [B, P].  Returns next_tok (int32 CUDA tensor [B])."""
        B, P = tokens.shape
        if next_tok is None:
            next_tok = self.torch.empty(B, dtype=self.torch.int32, device=self.device)
        _check(self.lib.d3_prefill(self.ctx, tokens.data_ptr(), B, P, pos_begin, next_tok.data_ptr(), _ptr(logits),
                                   _ptr(hidden_dump), self._stream()))
        return next_tok

    def prefill_ragged(self, tokens, lengths, next_tok=None, logits=None, hidden_dump=None):
        """tokens: int32 CUDA tensor [B, P], left-padded; lengths: B host ints (the longest equals P)."""
        B, P = tokens.shape
        lens = np.ascontiguousarray(lengths, np.int32)
        if lens.shape != (B,):
            raise ValueError("lengths must hold one entry per sequence")
        if next_tok is None:
            next_tok = self.torch.empty(B, dtype=self.torch.int32, device=self.device)
        _check(self.lib.d3_prefill_ragged(self.ctx, tokens.data_ptr(), lens.ctypes.data, B, P, next_tok.data_ptr(),
                                          _ptr(logits), _ptr(hidden_dump), self._stream()))
        return next_tok

    def decode_step(self, tok_in, step_i: int, tok_out, logits=None, hidden_dump=None) -> None:
        _check(self.lib.d3_decode_step(self.ctx, tok_in.data_ptr(), step_i, tok_out.data_ptr(), _ptr(logits),
                                       _ptr(hidden_dump), self._stream()))

    def decode_step_static(self, tok_in, step_i: int, tok_out, logits=None, hidden_dump=None) -> None:
        """decode_step with its intermediates in the library's static scratch array (no workspace use, no allocation)."""
        _check(self.lib.d3_decode_step_static(self.ctx, tok_in.data_ptr(), step_i, tok_out.data_ptr(), _ptr(logits),
                                              _ptr(hidden_dump), self._stream()))

    def fill_missing_kv(self, pos_begin: int, pos_end: int, mode: int = D3_FILL_COPY) -> None:
        _check(self.lib.d3_fill_missing_kv(self.ctx, pos_begin, pos_end, mode, self._stream()))

    def set_fill_mode(self, mode: int) -> None:
        _check(self.lib.d3_set_fill_mode(self.ctx, mode))

    def synchronize(self) -> None:
        self.torch.cuda.current_stream(self.device).synchronize()

    def truncate(self, n_rows: int) -> None:
        _check(self.lib.d3_truncate(self.ctx, n_rows))

    def stream_read(self, tensor) -> None:
        """Read-only streaming yardstick over a CUDA tensor (one launch, asynchronous)."""
        _check(self.lib.d3_stream_read(self.ctx, tensor.data_ptr(), tensor.numel() * tensor.element_size(), self._stream()))

    def mfma_yardstick(self, mode: int, stages: int) -> None:
        """Matrix-core yardstick of the prompt pass (one launch, asynchronous): mode 0 MFMAs alone, 1 with the stage loop's
        LDS reads, 2 with its barrier too; n_cu workgroups x 8 waves x stages x 32 instructions of 16384 flops."""
        _check(self.lib.d3_mfma_yardstick(self.ctx, mode, stages, self._stream()))

    def profile_select(self, kernel_class: int) -> None:
        _check(self.lib.d3_profile_select(self.ctx, kernel_class))

    def profile_read(self):
        """(summed milliseconds, launches) of the selected kernel class since the last read."""
        ms, n = C.c_double(), C.c_int64()
        _check(self.lib.d3_profile_read(self.ctx, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    @property
    def n_ctx(self) -> int:
        return int(self.lib.d3_n_ctx(self.ctx))


def weights_to_device(shape, weights_np: Dict[str, object], device: str = "cuda:0") -> Dict[str, object]:
    """numpy weights (float32, or uint16 bf16 bit patterns) -> torch CUDA tensors, bit-exact."""
    import torch

    def conv(a: np.ndarray):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
        return torch.from_numpy(a).to(device)

    out = {k: conv(v) for k, v in weights_np.items() if k != "layers"}
    out["layers"] = [{k: conv(v) for k, v in lw.items()} for lw in weights_np["layers"]]
    return out


def random_weights_on_device(shape, seed: int = 0, device: str = "cuda:0") -> Dict[str, object]:
    """N(0, 0.02) weights drawn on the GPU (performance runs only: not bit-reproducible on the host)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    tdt = torch.float32 if shape.dtype == "f32" else torch.bfloat16

    def normal(*dims):
        t = torch.empty(dims, dtype=torch.float32, device=device)
        t.normal_(0.0, 0.02, generator=g)
        return t.to(tdt)

    s = shape
    layers = []
    for _ in range(s.L):
        layers.append({
            "attn_norm": torch.ones(s.d, dtype=torch.float32, device=device),
            "wq": normal(s.H * s.hd, s.d), "wk": normal(s.H_kv * s.hd, s.d), "wv": normal(s.H_kv * s.hd, s.d),
            "wo": normal(s.d, s.H * s.hd), "mlp_norm": torch.ones(s.d, dtype=torch.float32, device=device),
            "w_gate": normal(s.F, s.d), "w_up": normal(s.F, s.d), "w_down": normal(s.d, s.F)})
    return {"tok_emb": normal(s.V, s.d), "lm_head": normal(s.V, s.d),
            "final_norm": torch.ones(s.d, dtype=torch.float32, device=device), "layers": layers}
