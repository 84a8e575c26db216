"""ctypes wrapper over oracle/liboracle.so -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.  It does
argument marshalling and nothing else; the arithmetic is in adadecode_oracle.c.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

MAX_EXIT = 8
EV_LAYER_STEP, EV_HEAD, EV_VERIFY, EV_VERIFY_ROW = 1, 2, 3, 4


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rope_base", C.c_double), ("rms_eps", C.c_double), ("wdtype", C.c_int32),
                ("n_exit", C.c_int32), ("exit_layers", C.c_int32 * MAX_EXIT), ("kv_dtype", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class TopWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("exit_T", C.c_void_p * MAX_EXIT)]


class Event(C.Structure):
    _fields_ = [("kind", C.c_int32), ("layer", C.c_int32), ("pos", C.c_int32), ("m", C.c_int32),
                ("token", C.c_int32), ("flag", C.c_int32), ("conf", C.c_double), ("margin", C.c_double)]


EVENT_DTYPE = np.dtype([("kind", "<i4"), ("layer", "<i4"), ("pos", "<i4"), ("m", "<i4"), ("token", "<i4"),
                        ("flag", "<i4"), ("conf", "<f8"), ("margin", "<f8")])
assert EVENT_DTYPE.itemsize == C.sizeof(Event)


class GenParams(C.Structure):
    _fields_ = [("gamma", C.c_double), ("max_pending", C.c_int32), ("max_new", C.c_int32), ("eos_id", C.c_int32),
                ("forced_exit", C.c_void_p), ("scripted_draft", C.c_void_p),
                ("temperature", C.c_double), ("uniforms", C.c_void_p), ("head_mask", C.c_int32), ("no_verify", C.c_int32),
                ("keep_cache", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("tokens", "layer_steps", "layer_step_rows", "head_evals", "verifies",
                                         "early_preds", "rejections", "rolled_back")] + [("steps_by_m", C.c_int64 * 9)]

    def as_dict(self) -> dict:
        out = {n: int(getattr(self, n)) for n, _ in self._fields_[:-1]}
        out["steps_by_m"] = [int(x) for x in self.steps_by_m]
        return out


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        P = C.c_void_p
        i32, f64 = C.c_int32, C.c_double
        L.orc_model_new.restype = P
        L.orc_model_new.argtypes = [C.POINTER(Config), C.POINTER(LayerWeights), C.POINTER(TopWeights)]
        L.orc_model_free.argtypes = [P]
        L.orc_kv_new.restype = P
        L.orc_kv_new.argtypes = [P, i32]
        L.orc_kv_free.argtypes = [P]
        L.orc_kv_len.restype = i32
        L.orc_kv_len.argtypes = [P, i32]
        L.orc_kv_set_len.argtypes = [P, i32, i32]
        L.orc_kv_truncate.argtypes = [P, i32]
        L.orc_kv_write.argtypes = [P, i32, i32, i32, P, P]
        L.orc_kv_read.argtypes = [P, i32, i32, i32, P, P]
        L.orc_rmsnorm.argtypes = [P, P, i32, i32, f64, P]
        L.orc_rope.argtypes = [P, i32, i32, f64]
        L.orc_confidence.argtypes = [P, i32, P, P, P]
        L.orc_embed.argtypes = [P, P, i32, P]
        L.orc_layer_step.restype = C.c_int
        L.orc_layer_step.argtypes = [P, P, i32, P, P, i32]
        L.orc_head.argtypes = [P, i32, P, P, P, P, P]
        L.orc_verify.argtypes = [P, P, P, i32, P, P, P, P]
        L.orc_softmax_t.argtypes = [P, i32, f64, P]
        L.orc_sample_cdf.restype = i32
        L.orc_sample_cdf.argtypes = [P, i32, f64, P]
        L.orc_accept_or_resample.restype = C.c_int
        L.orc_accept_or_resample.argtypes = [P, P, i32, i32, f64, f64, P, P, P]
        L.orc_generate_greedy.restype = C.c_int
        L.orc_generate_greedy.argtypes = [P, P, P, i32, i32, i32, P, P, P]
        L.orc_generate_ada.restype = C.c_int
        L.orc_generate_ada.argtypes = [P, P, P, i32, C.POINTER(GenParams), P, P, C.POINTER(Stats), P, C.c_int64, P]
        L.orc_num_threads.restype = C.c_int
        L.orc_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]) -> Optional[int]:
    return None if a is None else a.ctypes.data


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


# --- stand-alone building blocks -------------------------------------------------------------------

def rmsnorm(x, w: np.ndarray, eps: float) -> np.ndarray:
    x = _f64(x)
    w = np.ascontiguousarray(w)
    assert w.dtype in (np.float32, np.uint16, np.float16)
    out = np.empty_like(x)
    lib().orc_rmsnorm(x.ctypes.data, w.ctypes.data, {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float16): 2}[w.dtype],
                      x.size, eps, out.ctypes.data)
    return out


def rope(vec, pos: int, base: float) -> np.ndarray:
    v = _f64(vec).copy()
    lib().orc_rope(v.ctypes.data, v.size, pos, base)
    return v


def confidence(z) -> Tuple[int, float, float]:
    z = _f64(z)
    tok, conf, margin = C.c_int32(), C.c_double(), C.c_double()
    lib().orc_confidence(z.ctypes.data, z.size, C.byref(tok), C.byref(conf), C.byref(margin))
    return tok.value, conf.value, margin.value


# --- model -----------------------------------------------------------------------------------------

class Oracle:
    """A model instance of the oracle over a synth.ModelShape and its weight dict."""

    def __init__(self, shape, weights: Dict[str, np.ndarray], max_pos: int, kv_dtype: Optional[int] = None):
        """kv_dtype: storage type of the oracle's KV cache (0 fp32 = unrounded fp64 values, 1 bf16, 2 fp16); by default
        the model's own type, as the workloads define it."""
        self.shape = shape
        self.weights = weights            # keeps the buffers alive
        self.L = lib()
        cfg = Config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                     shape.vocab, shape.rope_base, shape.rms_eps, shape.dtype, len(shape.exit_layers))
        for i, l in enumerate(shape.exit_layers):
            cfg.exit_layers[i] = l
        cfg.kv_dtype = shape.dtype if kv_dtype is None else kv_dtype   # a 16-bit workload keeps a KV cache of its type
        want = (np.float32, np.uint16, np.float16)[shape.dtype]
        for k, v in weights.items():
            assert v.dtype == want and v.flags["C_CONTIGUOUS"], k
        layers = (LayerWeights * shape.n_layers)()
        for l in range(shape.n_layers):
            for n, _ in LayerWeights._fields_:
                setattr(layers[l], n, weights[f"layers.{l}.{n}"].ctypes.data)
        top = TopWeights(weights["embed"].ctypes.data, weights["final_norm"].ctypes.data, weights["lm_head"].ctypes.data)
        for i in range(len(shape.exit_layers)):
            t = weights.get(f"exit_T.{i}")
            top.exit_T[i] = None if t is None else t.ctypes.data
        self.cfg = cfg
        self.model = self.L.orc_model_new(C.byref(cfg), layers, C.byref(top))
        if not self.model:
            raise ValueError("oracle rejected the configuration")
        self.max_pos = max_pos
        self.kv = self.L.orc_kv_new(self.model, max_pos)

    def close(self) -> None:
        if self.kv:
            self.L.orc_kv_free(self.kv)
            self.kv = None
        if self.model:
            self.L.orc_model_free(self.model)
            self.model = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # cache
    def kv_len(self, layer: int) -> int:
        return self.L.orc_kv_len(self.kv, layer)

    def kv_lens(self) -> List[int]:
        return [self.kv_len(l) for l in range(1, self.shape.n_layers + 1)]

    def kv_set_len(self, layer: int, n: int) -> None:
        self.L.orc_kv_set_len(self.kv, layer, n)

    def kv_truncate(self, n: int) -> None:
        self.L.orc_kv_truncate(self.kv, n)

    def kv_write(self, layer: int, pos0: int, k: np.ndarray, v: np.ndarray) -> None:
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        self.L.orc_kv_write(self.kv, layer, pos0, k.shape[0], k.ctypes.data, v.ctypes.data)

    def kv_read(self, layer: int, pos0: int, n: int) -> Tuple[np.ndarray, np.ndarray]:
        s = self.shape
        k = np.empty((n, s.n_kv_heads, s.head_dim), dtype=np.float64)
        v = np.empty_like(k)
        self.L.orc_kv_read(self.kv, layer, pos0, n, k.ctypes.data, v.ctypes.data)
        return k, v

    # steps
    def embed(self, tokens) -> np.ndarray:
        t = _i32(tokens)
        h = np.empty((t.size, self.shape.d_model), dtype=np.float64)
        self.L.orc_embed(self.model, t.ctypes.data, t.size, h.ctypes.data)
        return h

    def layer_step(self, layer: int, hidden: np.ndarray, pos) -> np.ndarray:
        h = _f64(hidden).copy()
        p = _i32(pos)
        assert h.shape == (p.size, self.shape.d_model)
        rc = self.L.orc_layer_step(self.model, self.kv, layer, h.ctypes.data, p.ctypes.data, p.size)
        if rc != 0:
            raise RuntimeError(f"orc_layer_step rc={rc}")
        return h

    def head(self, head_index: int, h, want_logits: bool = False):
        h = _f64(h)
        tok, conf, margin = C.c_int32(), C.c_double(), C.c_double()
        z = np.empty(self.shape.vocab, dtype=np.float64) if want_logits else None
        self.L.orc_head(self.model, head_index, h.ctypes.data, C.byref(tok), C.byref(conf), C.byref(margin), _ptr(z))
        return (tok.value, conf.value, margin.value, z) if want_logits else (tok.value, conf.value, margin.value)

    def verify(self, hidden, draft):
        h = _f64(hidden)
        m = h.shape[0]
        dr = _i32(draft) if m > 1 else np.zeros(1, dtype=np.int32)
        assert m == 1 or dr.size == m - 1
        n_acc, nxt = C.c_int32(), C.c_int32()
        arg = np.empty(m, dtype=np.int32)
        mar = np.empty(m, dtype=np.float64)
        self.L.orc_verify(self.model, h.ctypes.data, dr.ctypes.data, m, C.byref(n_acc), C.byref(nxt), arg.ctypes.data, mar.ctypes.data)
        return n_acc.value, nxt.value, arg, mar

    # generation
    def generate_greedy(self, prompt, max_new: int, eos_id: int = -1):
        p = _i32(prompt)
        out = np.empty(max_new, dtype=np.int32)
        mar = np.empty(max_new, dtype=np.float64)
        n = C.c_int32()
        rc = self.L.orc_generate_greedy(self.model, self.kv, p.ctypes.data, p.size, max_new, eos_id, out.ctypes.data,
                                        C.byref(n), mar.ctypes.data)
        if rc != 0:
            raise RuntimeError(f"orc_generate_greedy rc={rc}")
        return out[:n.value].copy(), mar[:n.value].copy()

    def generate_ada(self, prompt, max_new: int, gamma: float, max_pending: int = 5, eos_id: int = -1,
                     forced_exit: Optional[np.ndarray] = None, scripted_draft: Optional[np.ndarray] = None,
                     max_events: int = 1 << 20, temperature: float = 0.0, uniforms: Optional[np.ndarray] = None,
                     head_mask: int = 0, no_verify: bool = False, keep_cache: int = 0):
        """temperature > 0: sampled decoding with the draws `uniforms`, float32 [max_pos, n_exit + 3].
        head_mask / no_verify: the ablation switches (bit i enables exit head i; drafts are kept unchecked).
        keep_cache: leading prompt positions whose cache rows an earlier run on the same leading tokens left behind."""
        p = _i32(prompt)
        if temperature > 0:
            uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
            assert uniforms.shape == (self.max_pos, len(self.shape.exit_layers) + 3)
        if forced_exit is not None:
            forced_exit = np.ascontiguousarray(forced_exit, dtype=np.uint8)
            assert forced_exit.size >= self.max_pos
        if scripted_draft is not None:
            scripted_draft = _i32(scripted_draft)
            assert scripted_draft.size >= self.max_pos
        gp = GenParams(gamma, max_pending, max_new, eos_id, _ptr(forced_exit), _ptr(scripted_draft), temperature,
                       _ptr(uniforms) if temperature > 0 else None, head_mask, int(no_verify), int(keep_cache))
        out = np.empty(max_new + max_pending + 2, dtype=np.int32)
        ev = np.zeros(max_events, dtype=EVENT_DTYPE)
        n, nev, st = C.c_int32(), C.c_int64(), Stats()
        rc = self.L.orc_generate_ada(self.model, self.kv, p.ctypes.data, p.size, C.byref(gp), out.ctypes.data, C.byref(n),
                                     C.byref(st), ev.ctypes.data, max_events, C.byref(nev))
        if rc != 0:
            raise RuntimeError(f"orc_generate_ada rc={rc}")
        assert nev.value <= max_events, "event buffer too small"
        return out[:n.value].copy(), st.as_dict(), ev[:nev.value].copy()


def softmax_t(z, temperature: float) -> np.ndarray:
    z = np.ascontiguousarray(z, dtype=np.float64)
    p = np.empty_like(z)
    lib().orc_softmax_t(z.ctypes.data, z.size, C.c_double(temperature), p.ctypes.data)
    return p


def sample_cdf(w, u: float):
    """(token, margin) of the inversion draw u over the weights w."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    mg = C.c_double()
    t = lib().orc_sample_cdf(w.ctypes.data, w.size, C.c_double(u), C.byref(mg))
    return int(t), mg.value


def accept_or_resample(p, q, t: int, u_accept: float, u_resample: float):
    """Eq. 2 for one drafted token: (accepted, replacement or -1, ratio, margin)."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    assert p.size == q.size
    repl, ratio, mg = C.c_int32(-1), C.c_double(), C.c_double()
    acc = lib().orc_accept_or_resample(p.ctypes.data, q.ctypes.data, p.size, t, C.c_double(u_accept), C.c_double(u_resample),
                                       C.byref(repl), C.byref(ratio), C.byref(mg))
    return bool(acc), int(repl.value), ratio.value, mg.value


def num_threads() -> int:
    return lib().orc_num_threads()


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(int(n))
