"""Seeded synthetic inputs: model shapes, random-init weights, prompts, forced exit schedules.

This module is data only. It serves both the CPU oracle (tests) and the HIP library (tests, bench,
smoke) with the *same* buffers, and contains none of the method's arithmetic: no norm, no attention,
no head, no scheduling.  The only numeric helpers are the storage roundings of fp32 values to bf16 bit
patterns and to IEEE half precision (both round-to-nearest-even), which is how the 16-bit workloads'
weights are defined.

The workloads stand in for the paper's models (Llama-3.1-8B-Instruct, CodeLlama-13B-Instruct; Sec. 3
"Experimental setup", Table 4 for the LM-head shapes) which are not available here: Llama-shaped
decoders with N(0, 0.02) weights, residual-branch output matrices scaled by 0.05.
"""
from __future__ import annotations

import concurrent.futures as _cf
import dataclasses
import hashlib
import os
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F32 = 0
BF16 = 1
F16 = 2     # IEEE half precision, the inference precision the paper reports (Sec. 4.2)


@dataclasses.dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    exit_layers: Tuple[int, ...]      # 1-based layer indices that carry an exit head, each < n_layers
    dtype: int                        # F32, BF16 or F16 (storage type of weights and of the KV cache)
    tied_head: bool                   # LM head shares the embedding matrix
    rms_eps: float = 1e-5
    gamma: float = 0.9
    prompt_len: int = 32
    gen_len: int = 64

    @property
    def d_q(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def layer_weight_elems(self) -> int:
        d, f = self.d_model, self.d_ffn
        return (self.d_q + 2 * self.d_kv) * d + d * self.d_q + 3 * d * f

    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    def with_(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


# The five workloads of the build's benchmark definition.  "tiny" is the fp32 parity model, "8b" and
# "13b" follow the LM-head shapes the paper lists in Table 4 (128256 x 4096, 32016 x 5120).
TINY = ModelShape("tiny", 4, 256, 4, 4, 64, 688, 2048, 10000.0, (2,), F32, True,
                  prompt_len=32, gen_len=64)
LLAMA8B = ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0, (8, 16, 24), BF16, False,
                     prompt_len=256, gen_len=1024)
LLAMA8B_LAYER = LLAMA8B.with_(name="8b-layer", n_layers=1, exit_layers=(), vocab=256)
LLAMA13B = ModelShape("13b", 40, 5120, 40, 40, 128, 13824, 32016, 10000.0, (10, 20, 30), BF16, False,
                      prompt_len=512, gen_len=1024)
LLAMA8B_LONG = LLAMA8B.with_(name="8b-long", prompt_len=1024, gen_len=8192)

# Reduced-depth variants used where the full model would make a CPU comparison take too long; the
# per-layer shapes (what every kernel sees) are unchanged.
TINY_BF16 = TINY.with_(name="tiny-bf16", dtype=BF16)
TINY_F16 = TINY.with_(name="tiny-f16", dtype=F16)
TINY_GQA = TINY.with_(name="tiny-gqa", n_q_heads=4, n_kv_heads=2, n_layers=6, exit_layers=(2, 4))
MINI8B = LLAMA8B.with_(name="8b-mini", n_layers=4, exit_layers=(1, 2, 3), vocab=8192,
                       prompt_len=24, gen_len=24)
MINI13B = LLAMA13B.with_(name="13b-mini", n_layers=4, exit_layers=(1, 2, 3), vocab=4016,
                         prompt_len=24, gen_len=24)

# A d_model = 8192 decoder, the width of the largest LM head the paper lists in Table 4 (32000 x 8192), in
# the paper's inference precision.  The paper does not print that model's head counts or FFN width: the values
# here are stand-ins chosen for this workload, not that model's.
WIDE_LAYER = ModelShape("wide-layer", 1, 8192, 64, 16, 128, 20480, 256, 10000.0, (), F16, False,
                        prompt_len=16, gen_len=16)
WIDE_MINI = WIDE_LAYER.with_(name="wide-mini", n_layers=3, exit_layers=(1, 2), vocab=4000)

SHAPES = {s.name: s for s in (TINY, LLAMA8B, LLAMA8B_LAYER, LLAMA13B, LLAMA8B_LONG, TINY_BF16, TINY_F16,
                              TINY_GQA, MINI8B, MINI13B, WIDE_LAYER, WIDE_MINI)}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def store_as(x: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 values in the storage type of a workload: fp32 as is, bf16 as uint16 bit patterns, fp16 as numpy
    float16 (numpy's conversion rounds to nearest even)."""
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(x)
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _tensor_seed(seed: int, name: str) -> np.random.Generator:
    h = hashlib.sha256(f"{seed}:{name}".encode()).digest()
    return np.random.default_rng(int.from_bytes(h[:16], "little"))


def _normal(seed: int, name: str, shape: Sequence[int], std: float, dtype: int) -> np.ndarray:
    rng = _tensor_seed(seed, name)
    n = int(np.prod(shape))
    out = np.empty(n, dtype={F32: np.float32, BF16: np.uint16, F16: np.float16}[dtype])
    step = 1 << 24
    for s in range(0, n, step):        # chunked so that the fp32 temporary stays small
        e = min(n, s + step)
        blk = rng.standard_normal(e - s, dtype=np.float32)
        blk *= np.float32(std)
        out[s:e] = store_as(blk, dtype)
    return out.reshape(shape)


def _ones(shape: Sequence[int], dtype: int) -> np.ndarray:
    return store_as(np.ones(shape, dtype=np.float32), dtype)


def make_weights(shape: ModelShape, seed: int = 0, *, with_T: bool = False, T_std: float = 0.01,
                 norm_jitter: float = 0.0, workers: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Random-init weights of a Llama-shaped decoder.

    All matrices are [out_features, in_features] row-major, N(0, 0.02); attention-output and FFN-down
    are scaled by 0.05.  Norm weights are 1 (or 1 + N(0, norm_jitter) when asked, so that tests see a
    non-trivial norm weight).  `with_T` adds one [d, d] transform per exit head, I + N(0, T_std), as a
    stand-in for the trained lightweight heads of Sec. 2.1.
    """
    d, f, dt = shape.d_model, shape.d_ffn, shape.dtype
    jobs: List[Tuple[str, Tuple[int, ...], float]] = [("embed", (shape.vocab, d), 0.02)]
    if not shape.tied_head:
        jobs.append(("lm_head", (shape.vocab, d), 0.02))
    for l in range(shape.n_layers):
        p = f"layers.{l}."
        jobs += [(p + "wq", (shape.d_q, d), 0.02), (p + "wk", (shape.d_kv, d), 0.02),
                 (p + "wv", (shape.d_kv, d), 0.02), (p + "wo", (d, shape.d_q), 0.02 * 0.05),
                 (p + "w_gate", (f, d), 0.02), (p + "w_up", (f, d), 0.02),
                 (p + "w_down", (d, f), 0.02 * 0.05)]
    if workers is None:
        workers = max(1, min(16, (os.cpu_count() or 1)))
    out: Dict[str, np.ndarray] = {}
    with _cf.ThreadPoolExecutor(max_workers=workers) as ex:
        futs = {name: ex.submit(_normal, seed, name, shp, std, dt) for name, shp, std in jobs}
        for name, fu in futs.items():
            out[name] = fu.result()
    if shape.tied_head:
        out["lm_head"] = out["embed"]

    def norm_w(name: str) -> np.ndarray:
        if norm_jitter == 0.0:
            return _ones((d,), dt)
        v = 1.0 + norm_jitter * _tensor_seed(seed, name).standard_normal(d).astype(np.float32)
        return store_as(v, dt)

    out["final_norm"] = norm_w("final_norm")
    for l in range(shape.n_layers):
        out[f"layers.{l}.attn_norm"] = norm_w(f"layers.{l}.attn_norm")
        out[f"layers.{l}.ffn_norm"] = norm_w(f"layers.{l}.ffn_norm")
    if with_T:
        for i, _ in enumerate(shape.exit_layers):
            t = T_std * _tensor_seed(seed, f"exit_T.{i}").standard_normal((d, d)).astype(np.float32)
            t += np.eye(d, dtype=np.float32)
            out[f"exit_T.{i}"] = store_as(t, dt)
    return out


def make_prompt(shape: ModelShape, seed: int = 0, n: Optional[int] = None) -> np.ndarray:
    n = shape.prompt_len if n is None else n
    return _tensor_seed(seed, "prompt").integers(0, shape.vocab, size=n, dtype=np.int32)


def make_hidden(shape: ModelShape, seed: int, m: int) -> np.ndarray:
    """[m, d] N(0,1) hidden rows (fp32), the layer-step microbenchmark's input."""
    return _tensor_seed(seed, "hidden").standard_normal((m, shape.d_model), dtype=np.float32)


# The single-layer microbenchmark: row counts, calls per row count, and the seed of call number `call` with m rows
# (every call draws its own hidden rows).
MICRO_M = (1, 2, 3, 4, 6, 8)
MICRO_CALLS = 1000


def micro_call_seed(m: int, call: int) -> int:
    return 100000 + 1000 * m + call


def make_kv_prefill(shape: ModelShape, seed: int, layer: int, n_pos: int) -> Tuple[np.ndarray, np.ndarray]:
    """K and V values for positions [0, n_pos) of one layer, each [n_pos, n_kv_heads, head_dim], N(0,1).

    For a 16-bit shape the values are already rounded to the cache's type (returned as fp32 holding exactly
    representable numbers) so that the GPU cache and the oracle's cache start from identical numbers.
    """
    shp = (n_pos, shape.n_kv_heads, shape.head_dim)
    k = _tensor_seed(seed, f"kv.{layer}.k").standard_normal(shp, dtype=np.float32)
    v = _tensor_seed(seed, f"kv.{layer}.v").standard_normal(shp, dtype=np.float32)
    if shape.dtype != F32:
        k = as_f32(store_as(k, shape.dtype))
        v = as_f32(store_as(v, shape.dtype))
    return k, v


def make_forced_schedule(shape: ModelShape, seed: int, n_pos: int,
                         probs: Optional[Sequence[float]] = None) -> np.ndarray:
    """uint8[n_pos]: 0 = run to full depth, else the 1-based exit layer forced for the token at that
    absolute position.  Default: each exit layer with probability 0.2, drawn once from the seed."""
    k = len(shape.exit_layers)
    if probs is None:
        probs = [0.2] * k
    assert len(probs) == k and sum(probs) <= 1.0 + 1e-12
    u = _tensor_seed(seed, "forced").random(n_pos)
    out = np.zeros(n_pos, dtype=np.uint8)
    lo = 0.0
    for p, layer in zip(probs, shape.exit_layers):
        out[(u >= lo) & (u < lo + p)] = layer
        lo += p
    return out


def make_uniforms(shape: ModelShape, seed: int, n_pos: int) -> np.ndarray:
    """float32[n_pos, n_exit + 3] uniform draws in [0, 1) for sampled decoding, one row per absolute position:
    columns 0..n_exit-1 sample the position's successor at each exit head, column n_exit samples it at the final
    layer, column n_exit + 1 decides the acceptance of the token drafted after the position, column n_exit + 2
    draws that token's replacement after a rejection."""
    u = _tensor_seed(seed, "uniforms").random((n_pos, len(shape.exit_layers) + 3), dtype=np.float32)
    return np.minimum(u, np.float32(1.0 - 2.0 ** -24))


def as_f32(w: np.ndarray) -> np.ndarray:
    """The real values a stored tensor represents (fp32 array), whatever its storage type."""
    return bf16_bits_to_f32(w) if w.dtype == np.uint16 else w.astype(np.float32, copy=False)   # float16 widens exactly
