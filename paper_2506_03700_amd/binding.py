"""Thin ctypes binding over libadadecode.so (C ABI in include/adadecode.h).

Argument marshalling only: every step of the path runs in the library's kernels.  PyTorch supplies the
device buffers and the stream.  There is no CPU fallback: if the library is missing, importing the
functions fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libadadecode.so")
SCHED_TEST_LIB_PATH = os.path.join(HERE, "libad_sched_test.so")

AD_OK, AD_EINVAL, AD_ERANGE, AD_ESTATE, AD_EDEVICE, AD_ENOMEM = range(6)
AD_F32, AD_BF16, AD_F16 = 0, 1, 2
AD_MAX_EXIT, AD_M_MAX = 8, 8
EV_LAYER_STEP, EV_HEAD, EV_VERIFY, EV_VERIFY_ROW = 1, 2, 3, 4
AD_LAYER_KERNELS, AD_LAYER_FUSED = 0, 1
AD_PROF_GEMM, AD_PROF_LAYER = 0, 1
AD_PROBE_ONE_KERNEL, AD_PROBE_PER_PHASE = 0, 1

EXPORTS = ["ad_workspace_bytes", "ad_model_create", "ad_model_destroy", "ad_kv_bytes", "ad_kv_create", "ad_kv_destroy",
           "ad_kv_len", "ad_kv_set_len", "ad_kv_truncate", "ad_embed", "ad_layer_step", "ad_layer_steps", "ad_set_layer_mode", "ad_exit_head", "ad_verify",
           "ad_verify_static",
           "ad_head_logits", "ad_sample_logits", "ad_verify_sampled", "ad_generate", "ad_layer_trace", "ad_profile_start", "ad_profile_stop", "ad_probe_stream",
           "ad_last_error", "ad_version"]


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rope_base", C.c_float),
                ("rms_eps", C.c_float), ("dtype", C.c_int32), ("n_exit", C.c_int32),
                ("exit_layers", C.c_int32 * AD_MAX_EXIT), ("m_max", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class TopWeights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p), ("exit_T", C.POINTER(C.c_void_p))]


class GenParams(C.Structure):
    _fields_ = [("gamma", C.c_float), ("max_pending", C.c_int32), ("max_new", C.c_int32), ("eos_id", C.c_int32),
                ("forced_exit", C.c_void_p), ("scripted_draft", C.c_void_p), ("temperature", C.c_float), ("uniforms", C.c_void_p),
                ("head_mask", C.c_int32), ("no_verify", C.c_int32), ("no_issue_ahead", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("tokens", "layer_steps", "layer_step_rows", "head_evals", "verifies", "early_preds",
                                         "rejections", "rolled_back")] + \
               [("steps_by_m", C.c_int64 * (AD_M_MAX + 1)), ("bytes_algorithmic", C.c_int64)]

    def as_dict(self) -> dict:
        out = {n: int(getattr(self, n)) for n, t in self._fields_ if t is C.c_int64}
        out["steps_by_m"] = [int(x) for x in self.steps_by_m]
        return out


EVENT_DTYPE = np.dtype([("kind", "<i4"), ("layer", "<i4"), ("pos", "<i4"), ("m", "<i4"), ("token", "<i4"), ("flag", "<i4"),
                        ("conf", "<f4"), ("reserved", "<f4")])


class AdError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"status {status}: {text}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Loads the HIP library.  Raises if it has not been built: there is no other implementation."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_03700_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback path")
        L = C.CDLL(LIB_PATH)
        P, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
        L.ad_workspace_bytes.restype = sz
        L.ad_workspace_bytes.argtypes = [C.POINTER(Config)]
        L.ad_model_create.argtypes = [C.POINTER(Config), C.POINTER(LayerWeights), C.POINTER(TopWeights), P, sz, P, C.POINTER(P)]
        L.ad_model_destroy.argtypes = [P]
        L.ad_kv_bytes.restype = sz
        L.ad_kv_bytes.argtypes = [C.POINTER(Config), i32]
        L.ad_kv_create.argtypes = [P, P, sz, i32, P, C.POINTER(P)]
        L.ad_kv_destroy.argtypes = [P]
        L.ad_kv_len.argtypes = [P, i32, C.POINTER(i32)]
        L.ad_kv_set_len.argtypes = [P, i32, i32]
        L.ad_kv_truncate.argtypes = [P, i32]
        L.ad_embed.argtypes = [P, P, i32, P, P]
        L.ad_layer_step.argtypes = [P, P, i32, P, P, i32, P]
        L.ad_layer_steps.argtypes = [P, P, i32, i32, P, P, i32, P]
        L.ad_exit_head.argtypes = [P, i32, P, P, P, P]
        L.ad_verify.argtypes = [P, P, P, i32, P, P, P, P]
        L.ad_verify_static.argtypes = [P, P, P, i32, P, P, P, P]
        L.ad_head_logits.argtypes = [P, i32, P, i32, P, P]
        L.ad_sample_logits.argtypes = [P, P, C.c_float, C.c_float, P, P, P]
        L.ad_verify_sampled.argtypes = [P, P, P, P, i32, C.c_float, P, P, C.c_float, P, P, P, P]
        L.ad_generate.argtypes = [P, P, P, i32, C.POINTER(GenParams), P, P, C.POINTER(Stats), P, C.c_int64, P, P]
        L.ad_profile_start.argtypes = [P, i32, i32, i32]
        L.ad_set_layer_mode.argtypes = [P, i32]
        L.ad_layer_trace.argtypes = [P, P, C.c_size_t, P, P]
        L.ad_profile_stop.argtypes = [P, P, P, P, P, P]
        L.ad_probe_stream.argtypes = [P, P, i32, i32, i32, P]
        L.ad_last_error.restype = C.c_char_p
        L.ad_version.restype = C.c_char_p
        for n in EXPORTS:
            if n not in ("ad_workspace_bytes", "ad_kv_bytes", "ad_last_error", "ad_version"):
                getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != AD_OK:
        raise AdError(status, lib().ad_last_error().decode())


def make_config(shape, m_max: int = AD_M_MAX) -> Config:
    cfg = Config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                 shape.rope_base, shape.rms_eps, shape.dtype, len(shape.exit_layers))
    for i, l in enumerate(shape.exit_layers):
        cfg.exit_layers[i] = l
    cfg.m_max = m_max
    return cfg


def _stream_ptr(torch):
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Model:
    """ad_model + ad_kv over torch device buffers.  Method names follow the C entry points."""

    def __init__(self, shape, weights: Dict[str, np.ndarray], max_pos: int, m_max: int = AD_M_MAX, device: str = "cuda:0",
                 layer_mode: Optional[int] = None):
        import torch
        self.torch = torch
        self.shape = shape
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.L = lib()
        self.cfg = make_config(shape, m_max)
        ws_bytes = self.L.ad_workspace_bytes(C.byref(self.cfg))
        if ws_bytes == 0:
            raise AdError(AD_EINVAL, self.L.ad_last_error().decode())
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=self.device)
        self.model = C.c_void_p()
        self.kv = C.c_void_p()
        # stage the caller-side weights on the device one layer at a time; the library keeps its own copy
        layers = (LayerWeights * shape.n_layers)()
        keep = []

        def dev(a: np.ndarray):
            t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(self.device)
            keep.append(t)
            return t.data_ptr()

        for l in range(shape.n_layers):
            for n, _ in LayerWeights._fields_:
                setattr(layers[l], n, dev(weights[f"layers.{l}.{n}"]))
        top = TopWeights()
        top.embed = dev(weights["embed"])
        top.final_norm = dev(weights["final_norm"])
        top.lm_head = top.embed if weights["lm_head"] is weights["embed"] else dev(weights["lm_head"])
        tarr = (C.c_void_p * AD_MAX_EXIT)()
        any_T = False
        for i in range(len(shape.exit_layers)):
            t = weights.get(f"exit_T.{i}")
            if t is not None:
                tarr[i] = dev(t)
                any_T = True
        top.exit_T = C.cast(tarr, C.POINTER(C.c_void_p)) if any_T else None
        _check(self.L.ad_model_create(C.byref(self.cfg), layers, C.byref(top), C.c_void_p(self.workspace.data_ptr()), ws_bytes,
                                      _stream_ptr(torch), C.byref(self.model)))
        torch.cuda.synchronize()
        del keep          # the originals may be freed once creation has been synchronised
        self.max_pos = max_pos
        kv_bytes = self.L.ad_kv_bytes(C.byref(self.cfg), max_pos)
        self.kv_storage = torch.zeros(kv_bytes, dtype=torch.uint8, device=self.device)
        _check(self.L.ad_kv_create(self.model, C.c_void_p(self.kv_storage.data_ptr()), kv_bytes, max_pos, _stream_ptr(torch), C.byref(self.kv)))
        self._pinned = torch.zeros(64, dtype=torch.int32).pin_memory()
        if layer_mode is not None:
            self.ad_set_layer_mode(layer_mode)

    def close(self) -> None:
        if getattr(self, "kv", None):
            self.L.ad_kv_destroy(self.kv)
            self.kv = None
        if getattr(self, "model", None):
            self.torch.cuda.synchronize()
            self.L.ad_model_destroy(self.model)
            self.model = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- cache ----
    def kv_len(self, layer: int) -> int:
        n = C.c_int32()
        _check(self.L.ad_kv_len(self.kv, layer, C.byref(n)))
        return n.value

    def kv_lens(self) -> List[int]:
        return [self.kv_len(l) for l in range(1, self.shape.n_layers + 1)]

    def kv_set_len(self, layer: int, n: int) -> None:
        _check(self.L.ad_kv_set_len(self.kv, layer, n))

    def kv_truncate(self, n: int) -> None:
        _check(self.L.ad_kv_truncate(self.kv, n))

    @property
    def kv_stride(self) -> int:
        return (self.max_pos + 63) // 64 * 64

    def kv_views(self):
        """(K, V): K as [layer][kv head][position][head_dim], V as [layer][kv head][head_dim][position]
        (the library stores V transposed), positions 0..stride, of the storage dtype."""
        s, torch = self.shape, self.torch
        dt = {AD_F32: torch.float32, AD_BF16: torch.bfloat16, AD_F16: torch.float16}[s.dtype]
        half = s.n_kv_heads * self.kv_stride * s.head_dim
        flat = self.kv_storage[: s.n_layers * 2 * half * s.elem_bytes()].view(dt).view(s.n_layers, 2, half)
        k = flat[:, 0].view(s.n_layers, s.n_kv_heads, self.kv_stride, s.head_dim)
        v = flat[:, 1].view(s.n_layers, s.n_kv_heads, s.head_dim, self.kv_stride)
        return k, v

    def kv_fill(self, layer: int, k, v) -> None:
        """Write positions [0, n) of one layer from arrays [n, kv heads, head_dim] (benchmarks, tests)."""
        torch = self.torch
        K, V = self.kv_views()
        n = k.shape[0]
        K[layer - 1, :, :n, :] = torch.as_tensor(k).permute(1, 0, 2).to(K.device).to(K.dtype)
        V[layer - 1, :, :, :n] = torch.as_tensor(v).permute(1, 2, 0).to(V.device).to(V.dtype)

    def kv_read(self, layer: int, n: int):
        """Positions [0, n) of one layer as float64 numpy arrays [n, kv heads, head_dim]."""
        K, V = self.kv_views()
        k = K[layer - 1, :, :n, :].float().permute(1, 0, 2).cpu().numpy().astype(np.float64)
        v = V[layer - 1, :, :, :n].float().permute(2, 0, 1).cpu().numpy().astype(np.float64)
        return k, v

    # ---- steps (device tensors in, device tensors out) ----
    def ad_embed(self, tokens: Sequence[int]):
        torch = self.torch
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        h = torch.empty((t.size, self.shape.d_model), dtype=torch.float32, device=self.device)
        _check(self.L.ad_embed(self.model, t.ctypes.data, t.size, C.c_void_p(h.data_ptr()), _stream_ptr(torch)))
        return h

    def ad_layer_step(self, layer: int, hidden, pos: Sequence[int]) -> None:
        """In place on `hidden` (float32 [m, d], contiguous, on the model's device)."""
        torch = self.torch
        p = np.ascontiguousarray(pos, dtype=np.int32)
        assert hidden.dtype == torch.float32 and hidden.is_contiguous() and hidden.device == self.device
        assert hidden.shape == (p.size, self.shape.d_model)
        _check(self.L.ad_layer_step(self.model, self.kv, layer, C.c_void_p(hidden.data_ptr()), p.ctypes.data, p.size, _stream_ptr(torch)))

    def ad_layer_steps(self, first_layer: int, n_layers: int, hidden, pos: Sequence[int]) -> None:
        """Layers first_layer .. first_layer + n_layers - 1 over the same rows, in place on `hidden`."""
        torch = self.torch
        p = np.ascontiguousarray(pos, dtype=np.int32)
        assert hidden.dtype == torch.float32 and hidden.is_contiguous() and hidden.device == self.device
        assert hidden.shape == (p.size, self.shape.d_model)
        _check(self.L.ad_layer_steps(self.model, self.kv, first_layer, n_layers, C.c_void_p(hidden.data_ptr()), p.ctypes.data, p.size,
                                     _stream_ptr(torch)))

    def ad_exit_head(self, layer: int, hidden_row, sync: bool = True):
        """sync=False: only enqueues the evaluation (for timing launches back to back) and returns None."""
        torch = self.torch
        assert hidden_row.dtype == torch.float32 and hidden_row.is_contiguous() and hidden_row.numel() == self.shape.d_model
        out = self._pinned
        _check(self.L.ad_exit_head(self.model, layer, C.c_void_p(hidden_row.data_ptr()), C.c_void_p(out.data_ptr()),
                                   C.c_void_p(out.data_ptr() + 4), _stream_ptr(torch)))
        if not sync:
            return None
        torch.cuda.current_stream().synchronize()
        return int(out[0]), float(out[1:2].view(torch.float32)[0])

    def ad_verify(self, hidden, draft: Sequence[int], static: bool = False):
        """static: through ad_verify_static (the library's own static scratch, no allocation)."""
        torch = self.torch
        m = hidden.shape[0]
        assert hidden.dtype == torch.float32 and hidden.is_contiguous() and hidden.shape[1] == self.shape.d_model
        d = np.ascontiguousarray(draft, dtype=np.int32)
        assert d.size == m - 1
        dptr = d.ctypes.data if m > 1 else None
        out = self._pinned
        fn = self.L.ad_verify_static if static else self.L.ad_verify
        _check(fn(self.model, C.c_void_p(hidden.data_ptr()), dptr, m, C.c_void_p(out.data_ptr() + 32),
                  C.c_void_p(out.data_ptr() + 36), C.c_void_p(out.data_ptr() + 64), _stream_ptr(torch)))
        torch.cuda.current_stream().synchronize()
        return int(out[8]), int(out[9]), out[16:16 + m].numpy().copy()

    def ad_head_logits(self, layer: int, hidden):
        torch = self.torch
        m = hidden.shape[0]
        z = torch.empty((m, self.shape.vocab), dtype=torch.float32, device=self.device)
        _check(self.L.ad_head_logits(self.model, layer, C.c_void_p(hidden.data_ptr()), m, C.c_void_p(z.data_ptr()), _stream_ptr(torch)))
        return z

    def ad_sample_logits(self, logits, temperature: float, u: float):
        """(token, its probability) drawn from softmax(logits / temperature) with the uniform draw u."""
        torch = self.torch
        assert logits.dtype == torch.float32 and logits.is_contiguous() and logits.numel() == self.shape.vocab
        out = self._pinned
        _check(self.L.ad_sample_logits(self.model, C.c_void_p(logits.data_ptr()), temperature, u, C.c_void_p(out.data_ptr()),
                                       C.c_void_p(out.data_ptr() + 4), _stream_ptr(torch)))
        torch.cuda.current_stream().synchronize()
        return int(out[0]), float(out[1:2].view(torch.float32)[0])

    def ad_verify_sampled(self, final_logits, draft_logits, draft: Sequence[int], temperature: float, u_accept, u_resample,
                          u_final: float):
        """Eq. 2 on device logits: (n_accept, next_token, ratios[m-1])."""
        torch = self.torch
        m = final_logits.shape[0]
        V = self.shape.vocab
        assert final_logits.dtype == torch.float32 and final_logits.is_contiguous() and final_logits.shape[1] == V
        d = np.ascontiguousarray(draft, dtype=np.int32)
        ua = np.ascontiguousarray(u_accept, dtype=np.float32)
        ur = np.ascontiguousarray(u_resample, dtype=np.float32)
        assert d.size == ua.size == ur.size == m - 1
        if m > 1:
            assert draft_logits.dtype == torch.float32 and draft_logits.is_contiguous() and tuple(draft_logits.shape) == (m - 1, V)
        out = self._pinned
        _check(self.L.ad_verify_sampled(self.model, C.c_void_p(final_logits.data_ptr()),
                                        C.c_void_p(draft_logits.data_ptr()) if m > 1 else None,
                                        d.ctypes.data if m > 1 else None, m, temperature,
                                        ua.ctypes.data if m > 1 else None, ur.ctypes.data if m > 1 else None, u_final,
                                        C.c_void_p(out.data_ptr() + 32), C.c_void_p(out.data_ptr() + 36),
                                        C.c_void_p(out.data_ptr() + 64), _stream_ptr(torch)))
        torch.cuda.current_stream().synchronize()
        return int(out[8]), int(out[9]), out[16:16 + m - 1].view(torch.float32).numpy().copy()

    def ad_generate(self, prompt, max_new: int, gamma: float, max_pending: int = 5, eos_id: int = -1,
                    forced_exit: Optional[np.ndarray] = None, scripted_draft: Optional[np.ndarray] = None,
                    max_events: int = 1 << 20, want_events: bool = True, temperature: float = 0.0,
                    uniforms: Optional[np.ndarray] = None, head_mask: int = 0, no_verify: bool = False,
                    no_issue_ahead: bool = False):
        """temperature > 0: sampled decoding with the draws `uniforms`, float32 [max_pos, n_exit + 3].
        head_mask / no_verify: ablation switches (bit i enables exit head i; drafts are kept unchecked).
        no_issue_ahead: nothing is issued behind a head evaluation before its outcome is known."""
        torch = self.torch
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        if temperature > 0:
            uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
            assert uniforms.shape == (self.max_pos, len(self.shape.exit_layers) + 3)
        if forced_exit is not None:
            forced_exit = np.ascontiguousarray(forced_exit, dtype=np.uint8)
            assert forced_exit.size >= self.max_pos
        if scripted_draft is not None:
            scripted_draft = np.ascontiguousarray(scripted_draft, dtype=np.int32)
            assert scripted_draft.size >= self.max_pos
        gp = GenParams(gamma, max_pending, max_new, eos_id,
                       None if forced_exit is None else forced_exit.ctypes.data,
                       None if scripted_draft is None else scripted_draft.ctypes.data,
                       temperature, uniforms.ctypes.data if temperature > 0 else None, head_mask, int(no_verify),
                       int(no_issue_ahead))
        out = np.empty(max_new, dtype=np.int32)
        ev = np.zeros(max_events if want_events else 1, dtype=EVENT_DTYPE)
        n, nev, st = C.c_int32(), C.c_int64(), Stats()
        _check(self.L.ad_generate(self.model, self.kv, p.ctypes.data, p.size, C.byref(gp), out.ctypes.data, C.byref(n), C.byref(st),
                                  ev.ctypes.data if want_events else None, max_events if want_events else 0, C.byref(nev),
                                  _stream_ptr(torch)))
        return out[:n.value].copy(), st.as_dict(), ev[:min(nev.value, len(ev))].copy() if want_events else None


    def ad_set_layer_mode(self, mode: int) -> None:
        _check(self.L.ad_set_layer_mode(self.model, mode))

    def ad_layer_trace(self, on: bool = True):
        """Returns the device tensor [workgroups, stamps] (int64 ticks of the 100 MHz wall clock) that every fused
        layer-step launch overwrites from now on, or None after switching the trace off."""
        torch = self.torch
        nwg, ns = C.c_int32(), C.c_int32()
        _check(self.L.ad_layer_trace(self.model, None, 0, C.byref(nwg), C.byref(ns)))
        if not on:
            self._trace = None
            return None
        self._trace = torch.zeros((nwg.value, ns.value), dtype=torch.int64, device="cuda:0")
        _check(self.L.ad_layer_trace(self.model, self._trace.data_ptr(), self._trace.numel() * 8, None, None))
        return self._trace

    def ad_probe_stream(self, layer: int, ctx: int, mode: int) -> None:
        """Enqueues kernels that only read what one step of `layer` at context `ctx` must read (see the header)."""
        _check(self.L.ad_probe_stream(self.model, self.kv, layer, ctx, mode, _stream_ptr(self.torch)))

    def ad_profile_start(self, kind: int = AD_PROF_GEMM, period: int = 1, max_samples: int = 65536) -> None:
        _check(self.L.ad_profile_start(self.model, kind, period, max_samples))

    def ad_profile_stop(self) -> dict:
        nl, ns, sb, tb, ms = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64(), C.c_double()
        _check(self.L.ad_profile_stop(self.model, C.byref(nl), C.byref(ns), C.byref(ms), C.byref(sb), C.byref(tb)))
        return {"launches": nl.value, "samples": ns.value, "sampled_ms": ms.value, "sampled_bytes": sb.value, "total_bytes": tb.value}


# ---- CPU-only hook over the host scheduler (tests) ------------------------------------------------------

_sched = None


def sched_test_lib() -> C.CDLL:
    global _sched
    if _sched is None:
        L = C.CDLL(SCHED_TEST_LIB_PATH)
        P, i32 = C.c_void_p, C.c_int32
        L.ad_sched_test_run.restype = C.c_int
        L.ad_sched_test_run.argtypes = [i32, i32, P, i32, i32, i32, i32, i32, P, P, P, C.POINTER(GenParams), P, i32, P, P,
                                        C.POINTER(Stats), P, C.c_int64, P, P]
        L.ad_sched_test_stretches.restype = C.c_int64
        L.ad_sched_test_stretches.argtypes = [P, C.c_int64]
        L.ad_sched_test_hints.restype = C.c_int64
        L.ad_sched_test_hints.argtypes = [P, C.c_int64]
        _sched = L
    return _sched


def sched_test_stretches() -> np.ndarray:
    """The layer stretches the scheduler handed to the scripted backend in the last sched_test_run:
    rows of (first layer, layers, first row, rows, first position)."""
    L = sched_test_lib()
    n = L.ad_sched_test_stretches(None, 0)
    out = np.zeros((max(int(n), 1), 5), dtype=np.int32)
    L.ad_sched_test_stretches(out.ctypes.data, n)
    return out[:n]


def sched_test_hints() -> np.ndarray:
    """The hints the scheduler gave before the head evaluations of the last sched_test_run (what it would do next
    under the expected outcome): rows of (kind 1 = next layer / 2 = next token, layer, first row, rows, 1 if the
    calls after the evaluation asked for exactly that work)."""
    L = sched_test_lib()
    n = L.ad_sched_test_hints(None, 0)
    out = np.zeros((max(int(n), 1), 5), dtype=np.int32)
    L.ad_sched_test_hints(out.ctypes.data, n)
    return out[:n]


def sched_test_run(n_layers: int, exit_layers: Sequence[int], m_max: int, head_tok: np.ndarray, head_conf: np.ndarray,
                   final_tok: np.ndarray, prompt, max_new: int, gamma: float, max_pending: int, eos_id: int = -1,
                   forced_exit: Optional[np.ndarray] = None, scripted_draft: Optional[np.ndarray] = None, max_events: int = 1 << 18,
                   max_pos: Optional[int] = None, sequence: bool = False, temperature: float = 0.0,
                   uniforms: Optional[np.ndarray] = None, head_mask: int = 0, no_verify: bool = False, no_issue_ahead: bool = False):
    """Runs the library's host scheduler over scripted head outputs (no GPU).

    Table mode: head_tok/head_conf [max_pos, n_exit], final_tok [max_pos], looked up by position.
    Sequence mode: head_tok/head_conf are consumed one per head call, final_tok one per verified row."""
    L = sched_test_lib()
    ex = np.ascontiguousarray(exit_layers, dtype=np.int32)
    head_tok = np.ascontiguousarray(head_tok, dtype=np.int32)
    head_conf = np.ascontiguousarray(head_conf, dtype=np.float32)
    final_tok = np.ascontiguousarray(final_tok, dtype=np.int32)
    if not sequence:
        max_pos = final_tok.size
        assert head_tok.size == max_pos * max(1, ex.size) == head_conf.size
    assert max_pos is not None
    p = np.ascontiguousarray(prompt, dtype=np.int32)
    if forced_exit is not None:
        forced_exit = np.ascontiguousarray(forced_exit, dtype=np.uint8)
    if scripted_draft is not None:
        scripted_draft = np.ascontiguousarray(scripted_draft, dtype=np.int32)
    gp = GenParams(gamma, max_pending, max_new, eos_id, None if forced_exit is None else forced_exit.ctypes.data,
                   None if scripted_draft is None else scripted_draft.ctypes.data, temperature,
                   None if uniforms is None else uniforms.ctypes.data, head_mask, int(no_verify), int(no_issue_ahead))
    draws = np.full(4, -1.0, dtype=np.float32)
    out = np.empty(max_new + AD_M_MAX, dtype=np.int32)
    ev = np.zeros(max_events, dtype=EVENT_DTYPE)
    n, nev, st = C.c_int32(), C.c_int64(), Stats()
    rc = L.ad_sched_test_run(n_layers, ex.size, ex.ctypes.data, m_max, max_pos, int(sequence), head_tok.size, final_tok.size,
                             head_tok.ctypes.data, head_conf.ctypes.data,
                             final_tok.ctypes.data, C.byref(gp), p.ctypes.data, p.size, out.ctypes.data, C.byref(n), C.byref(st),
                             ev.ctypes.data, max_events, C.byref(nev), draws.ctypes.data)
    if temperature > 0:
        return rc, out[:max(0, n.value)].copy(), st.as_dict(), ev[:nev.value].copy(), draws
    return rc, out[:max(0, n.value)].copy(), st.as_dict(), ev[:nev.value].copy()
