"""ctypes front end of the C oracle.  TEST INFRASTRUCTURE ONLY: imported by the
tests, the smoke check and the benchmark's cpu_baseline leg, never by the
product package.

`generate` strings the oracle's steps together exactly as the method runs
(Section 3.1: prompt pass, then one token per step; Section 3.4: step i keeps
floor(L*alpha^i) blocks): the prompt goes through every block, token T_0 comes
from the last prompt position, and decode step i >= 1 feeds T_{i-1} at absolute
position P+i-1 through the blocks executed(i).
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("L", "d", "H", "H_kv", "hd", "F", "V")] + [
        ("eps", C.c_double), ("rope_base", C.c_double), ("weight_dtype", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")]


_LIBS = {}


def _lib(variant: str) -> C.CDLL:
    if variant not in _LIBS:
        _build.build()
        lib = C.CDLL(_build.lib_path(variant))
        i32, dbl, vp = C.c_int32, C.c_double, C.c_void_p
        lib.d3o_real_size.restype = C.c_int
        lib.d3o_set_threads.argtypes = [C.c_int]
        lib.d3o_plan_depth.argtypes = [i32, dbl, i32, i32, i32, vp, vp, vp]
        lib.d3o_plan_depth.restype = C.c_int
        lib.d3o_plan_depth_linear.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp]
        lib.d3o_plan_depth_linear.restype = C.c_int
        lib.d3o_model_new.argtypes = [C.POINTER(_Config), vp, C.POINTER(_Layer), vp, vp]
        lib.d3o_model_new.restype = vp
        lib.d3o_model_free.argtypes = [vp]
        lib.d3o_seq_new.argtypes = [vp, i32]
        lib.d3o_seq_new.restype = vp
        lib.d3o_seq_free.argtypes = [vp]
        lib.d3o_forward_token.argtypes = [vp, i32, i32, vp, i32, vp, vp]
        lib.d3o_forward_token.restype = C.c_int
        lib.d3o_first_block_kv.argtypes = [vp, i32, i32, i32]
        lib.d3o_first_block_kv.restype = C.c_int
        lib.d3o_argmax.argtypes = [vp, i32]
        lib.d3o_argmax.restype = i32
        lib.d3o_fill_missing_kv.argtypes = [vp, i32, i32, i32]
        lib.d3o_fill_missing_kv.restype = C.c_int
        lib.d3o_fill_recompute.argtypes = [vp, i32, i32, i32, vp]
        lib.d3o_fill_recompute.restype = C.c_int
        lib.d3o_get_kv.argtypes = [vp, i32, i32, vp, vp]
        lib.d3o_get_kv.restype = C.c_int
        lib.d3o_rmsnorm.argtypes = [vp, vp, i32, dbl, vp]
        lib.d3o_rope.argtypes = [vp, i32, i32, dbl]
        lib.d3o_softmax.argtypes = [vp, i32]
        lib.d3o_silu.argtypes = [dbl]
        lib.d3o_silu.restype = dbl
        lib.d3o_attention_head.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        _LIBS[variant] = lib
    return _LIBS[variant]


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def set_threads(n: int, variant: str = "f64") -> None:
    _lib(variant).d3o_set_threads(int(n))


def plan_depth(L: int, alpha: float, start: int, min_keep: int, n_steps: int, variant: str = "f64"):
    """(keep[n_steps], drop_begin[n_steps], layer_ids[n_steps][L]) as int32 arrays."""
    keep = np.zeros(n_steps, np.int32)
    drop = np.zeros(n_steps, np.int32)
    ids = np.zeros((n_steps, L), np.int32)
    rc = _lib(variant).d3o_plan_depth(L, float(alpha), start, min_keep, n_steps, _ptr(keep), _ptr(drop), _ptr(ids))
    if rc != 0:
        raise ValueError("d3o_plan_depth: invalid arguments")
    return keep, drop, ids


def plan_depth_linear(L: int, keep_first: int, keep_last: int, start: int, n_steps: int, variant: str = "f64"):
    """Linear decay from keep_first (step 0) to keep_last (last step); same three arrays as plan_depth."""
    keep = np.zeros(n_steps, np.int32)
    drop = np.zeros(n_steps, np.int32)
    ids = np.zeros((n_steps, L), np.int32)
    rc = _lib(variant).d3o_plan_depth_linear(L, keep_first, keep_last, start, n_steps, _ptr(keep), _ptr(drop), _ptr(ids))
    if rc != 0:
        raise ValueError("d3o_plan_depth_linear: invalid arguments")
    return keep, drop, ids


class OracleModel:
    """Borrows the weight arrays (numpy float32 / uint16 bf16 bits); keeps them alive."""

    def __init__(self, shape, weights, variant: str = "f64"):
        self.lib = _lib(variant)
        self.variant = variant
        self.shape = shape
        self.weights = weights
        wd = {"f32": 0, "bf16": 1}[shape.dtype]
        want = np.float32 if wd == 0 else np.uint16
        for name in ("tok_emb", "lm_head"):
            assert weights[name].dtype == want and weights[name].flags.c_contiguous, name
        cfg = _Config(shape.L, shape.d, shape.H, shape.H_kv, shape.hd, shape.F, shape.V,
                      float(shape.eps), float(shape.rope_base), wd)
        layers = (_Layer * shape.L)()
        for l, lw in enumerate(weights["layers"]):
            for name, _ in _Layer._fields_:
                arr = lw[name]
                assert arr.flags.c_contiguous
                assert arr.dtype == (np.float32 if name.endswith("norm") else want), name
                setattr(layers[l], name, _ptr(arr))
        assert weights["final_norm"].dtype == np.float32
        self.handle = self.lib.d3o_model_new(C.byref(cfg), _ptr(weights["tok_emb"]), layers,
                                             _ptr(weights["final_norm"]), _ptr(weights["lm_head"]))
        if not self.handle:
            raise ValueError("d3o_model_new rejected the configuration")

    def __del__(self):
        if getattr(self, "handle", None):
            self.lib.d3o_model_free(self.handle)
            self.handle = None

    def new_seq(self, max_seq: int) -> "OracleSeq":
        return OracleSeq(self, max_seq)


class OracleSeq:
    def __init__(self, model: OracleModel, max_seq: int):
        self.model = model
        self.max_seq = max_seq
        self.handle = model.lib.d3o_seq_new(model.handle, max_seq)
        if not self.handle:
            raise MemoryError("d3o_seq_new failed")

    def __del__(self):
        if getattr(self, "handle", None):
            self.model.lib.d3o_seq_free(self.handle)
            self.handle = None

    def forward_token(self, token: int, pos: int, layer_ids: Sequence[int], want_hidden=False, want_logits=False):
        s = self.model.shape
        ids = np.ascontiguousarray(layer_ids, dtype=np.int32)
        hidden = np.zeros((len(ids) + 1, s.d), np.float64) if want_hidden else None
        logits = np.zeros(s.V, np.float64) if want_logits else None
        rc = self.model.lib.d3o_forward_token(self.handle, int(token), int(pos), _ptr(ids), len(ids),
                                              _ptr(hidden) if want_hidden else None,
                                              _ptr(logits) if want_logits else None)
        if rc != 0:
            raise ValueError("d3o_forward_token: invalid arguments")
        return hidden, logits

    def first_block_kv(self, token: int, pos: int, layer: int) -> None:
        """Only the cache write of forward_token(token, pos, [layer])."""
        if self.model.lib.d3o_first_block_kv(self.handle, int(token), int(pos), int(layer)) != 0:
            raise ValueError("d3o_first_block_kv: invalid arguments")

    def fill_missing_kv(self, pos: int, drop_begin: int, n_drop: int) -> None:
        if self.model.lib.d3o_fill_missing_kv(self.handle, pos, drop_begin, n_drop) != 0:
            raise ValueError("d3o_fill_missing_kv: invalid arguments")

    def fill_recompute(self, pos: int, drop_begin: int, n_drop: int, h: np.ndarray) -> None:
        """RECOMPUTE fill of row pos from the hidden state h that entered the drop window."""
        h = np.ascontiguousarray(h, np.float64)
        if self.model.lib.d3o_fill_recompute(self.handle, pos, drop_begin, n_drop, _ptr(h)) != 0:
            raise ValueError("d3o_fill_recompute: invalid arguments")

    def get_kv(self, layer: int, pos: int):
        s = self.model.shape
        k = np.zeros(s.H_kv * s.hd, np.float64)
        v = np.zeros(s.H_kv * s.hd, np.float64)
        if self.model.lib.d3o_get_kv(self.handle, layer, pos, _ptr(k), _ptr(v)) != 0:
            raise ValueError("d3o_get_kv: invalid arguments")
        return k, v


def argmax(logits: np.ndarray, variant: str = "f64") -> int:
    logits = np.ascontiguousarray(logits, np.float64)
    return int(_lib(variant).d3o_argmax(_ptr(logits), logits.size))


class Generation:
    """Everything one sequence's run produced."""
    def __init__(self):
        self.tokens: List[int] = []          # T_0 .. T_{G-1} (the oracle's own greedy choice)
        self.fed: List[int] = []             # token actually fed at each decode step (forced or own)
        self.logits: List[np.ndarray] = []   # [V] per generated token
        self.hidden: List[np.ndarray] = []   # [(k_i+1), d] per generated token (last prompt row for i=0)
        self.keep = self.drop_begin = self.layer_ids = None
        self.seq: Optional[OracleSeq] = None
        self.n_rows = 0


def generate(model: OracleModel, prompt: Sequence[int], G: int, alpha: float, start: int, min_keep: int = 0,
             max_seq: Optional[int] = None, forced: Optional[Sequence[int]] = None,
             seq: Optional[OracleSeq] = None, pos_begin: int = 0, want_hidden: bool = True,
             plan=None) -> Generation:
    """Prompt pass + G-1 decode steps for one sequence.

    forced: if given, token fed at decode step i is forced[i-1] instead of the
    oracle's own T_{i-1} (teacher forcing; logits/tokens are still recorded).
    seq/pos_begin: continue on an existing cache whose rows [0, pos_begin) are set.
    plan: (keep, drop_begin, layer_ids) of G steps to follow instead of the power law (alpha, start, min_keep).
    """
    L = model.shape.L
    P = len(prompt)
    out = Generation()
    if plan is not None:
        out.keep, out.drop_begin, out.layer_ids = plan
    else:
        out.keep, out.drop_begin, out.layer_ids = plan_depth(L, alpha, start, min_keep, max(G, 1), model.variant)
    if seq is None:
        seq = model.new_seq(max_seq or (pos_begin + P + G))
    out.seq = seq
    all_layers = list(range(L))
    hidden = logits = None
    for t, tok in enumerate(prompt):          # initiation phase: every block, every prompt position
        last = t == P - 1
        hidden, logits = seq.forward_token(int(tok), pos_begin + t, all_layers, want_hidden and last, last)
    out.tokens.append(argmax(logits, model.variant))
    out.logits.append(logits)
    out.hidden.append(hidden)
    for i in range(1, G):                     # generation phase
        feed = int(forced[i - 1]) if forced is not None else out.tokens[i - 1]
        out.fed.append(feed)
        ids = out.layer_ids[i, : out.keep[i]]
        hidden, logits = seq.forward_token(feed, pos_begin + P + i - 1, ids, want_hidden, True)
        out.tokens.append(argmax(logits, model.variant))
        out.logits.append(logits)
        out.hidden.append(hidden)
    out.n_rows = pos_begin + P + G - 1
    return out


def fill_generated_rows(gen: Generation, P: int, G: int, pos_begin: int = 0, mode: str = "copy") -> None:
    """COPY (or RECOMPUTE) fill of every row written by decode steps 1..G-1 of `gen`.  RECOMPUTE needs the hidden
    states that generate() recorded: the state copied through a step's drop window is the one after the executed
    blocks that precede the window (the embedding when there are none)."""
    L = gen.seq.model.shape.L
    for i in range(1, G):
        s, n = int(gen.drop_begin[i]), int(L - gen.keep[i])
        if mode == "copy":
            gen.seq.fill_missing_kv(pos_begin + P + i - 1, s, n)
        else:
            before = int((gen.layer_ids[i, : gen.keep[i]] < s).sum())
            gen.seq.fill_recompute(pos_begin + P + i - 1, s, n, gen.hidden[i][before])


# ---- sub-functions (for the pins) ----

def rmsnorm(x, gain, eps, variant="f64"):
    x = np.ascontiguousarray(x, np.float64); gain = np.ascontiguousarray(gain, np.float32)
    out = np.zeros_like(x)
    _lib(variant).d3o_rmsnorm(_ptr(x), _ptr(gain), x.size, float(eps), _ptr(out))
    return out


def rope(vec, pos, base, variant="f64"):
    v = np.array(vec, np.float64, copy=True)
    _lib(variant).d3o_rope(_ptr(v), v.size, int(pos), float(base))
    return v


def softmax(v, variant="f64"):
    v = np.array(v, np.float64, copy=True)
    _lib(variant).d3o_softmax(_ptr(v), v.size)
    return v


def silu(x, variant="f64"):
    return float(_lib(variant).d3o_silu(float(x)))


def attention_head(q, K, V, variant="f64"):
    """q [hd], K/V [n_rows, hd] -> [hd]."""
    q = np.ascontiguousarray(q, np.float64); K = np.ascontiguousarray(K, np.float64); V = np.ascontiguousarray(V, np.float64)
    out = np.zeros(q.size, np.float64)
    _lib(variant).d3o_attention_head(_ptr(q), _ptr(K), _ptr(V), K.shape[0], q.size, K.shape[1], _ptr(out))
    return out


# ---- efficiency conversion (Section 4.1 "Evaluation Metrics": average layers -> FLOPs reduction) ----

def flops_reduction(L: int, avg_layers: float, d: int, V: int, params_per_block: int) -> float:
    """Full-depth cost over D^3 cost per output token, counting the lm_head
    (V*d multiply-adds) in units of one block's parameters."""
    h = V * d / params_per_block
    return (L + h) / (avg_layers + h)
