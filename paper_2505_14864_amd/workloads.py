"""Seeded synthetic inputs for the token-routed sparse FFN layer.

This module only draws random numbers and converts storage formats.  It holds
none of the layer's arithmetic, and it is the one module that both the GPU
path's callers and the CPU oracle's callers use, so that both sides see the
same bytes.

The paper trains on a Wikipedia dump with released Mixtral-8x7B /
LLaMA-MoE-3.5B weights (Sec. 5); neither is needed to time or check the layer,
whose cost depends on shapes and on the routing histogram only.  The inputs
here take the paper's sequence length (2048) and micro-batch structure and the
named models' layer shapes, and stand in for the dataset and the weights.

Recipe (every tensor has its own sub-stream, SeedSequence([seed, tag, part])):
  logits   N(0,1) + bias[e];  bias[e] = (e+1)^(-s) for the Zipf configs
  scores   N(0,1)                       (Mixture-of-Depths token scores)
  exit     Geometric(p) on {1,2,...}    (early-exit layer per token)
  x, dout  N(0,1)
  weights  N(0, 0.02^2)
bf16 tensors are rounded to nearest-even from the fp32 draw and handed out as
uint16 bit patterns; `widen_bf16` gives the exact fp32 value of those bits.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

_TAGS = {"logits": 1, "scores": 2, "exit": 3, "x": 4, "dout": 5, "Wg": 6, "Wu": 7, "Wd": 8}


@dataclass(frozen=True)
class Workload:
    name: str
    mode: str            # "moe" | "mod" | "early_exit"
    T: int
    H: int
    F: int
    E: int = 1
    k: int = 1
    dtype: str = "bf16"  # "f32" | "bf16"
    bias: tuple = ()     # explicit per-expert logit bias (moe)
    zipf_s: float = 0.0  # bias[e] = (e+1)^-s when > 0 (moe)
    B: int = 0           # sequences (mod)
    S: int = 0           # sequence length (mod)
    cap: int = 0         # selected tokens per sequence (mod)
    layers: int = 1      # stacked layers (early_exit)
    exit_p: float = 0.0  # geometric parameter (early_exit)
    seed: int = 0
    extra: dict = field(default_factory=dict, compare=False)


# The five benchmark configurations.
CONFIGS = {
    1: Workload("tiny_moe_f32", "moe", T=256, H=128, F=256, E=4, k=2, dtype="f32",
                bias=(1.0, 0.5, 0.0, -0.5), seed=1001),
    2: Workload("mixtral_8x7b_moe", "moe", T=4096, H=4096, F=14336, E=8, k=2, zipf_s=1.1, seed=1002),
    3: Workload("llama_moe_3p5b", "moe", T=8192, H=4096, F=688, E=16, k=4, zipf_s=1.3, seed=1003),
    4: Workload("mixture_of_depths", "mod", T=8192, H=2048, F=8192, B=4, S=2048, cap=256, seed=1004),
    5: Workload("early_exit_stack", "early_exit", T=16384, H=2048, F=8192, layers=4, exit_p=0.3, seed=1005),
}


def scaled(w: Workload, **kw) -> Workload:
    """The same recipe at other sizes (tests use small shapes)."""
    d = {f: getattr(w, f) for f in w.__dataclass_fields__ if f != "extra"}
    d.update(kw)
    return Workload(**d)


def _rng(seed, tag, part=0):
    return np.random.default_rng(np.random.SeedSequence([int(seed), _TAGS[tag], int(part)]))


def round_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the exact fp32 values."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK = 1 << 20  # elements drawn and converted at a time (keeps temporaries in cache)


def _normal(seed, tag, shape, sigma, dtype, part=0, out=None):
    """sigma * N(0,1) draws from the tensor's own sub-stream, in C order."""
    rng = _rng(seed, tag, part)
    n = int(np.prod(shape))
    if out is None:
        out = np.empty(shape, dtype=np.float32 if dtype == "f32" else np.uint16)
    flat = out.reshape(-1)
    sig = np.float32(sigma)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        a = rng.standard_normal(hi - lo, dtype=np.float32)
        if sigma != 1.0:
            a *= sig
        flat[lo:hi] = a if dtype == "f32" else round_to_bf16_bits(a)
    return out


def _per_part(seed, tag, parts, shape, sigma, dtype, threads):
    out = np.empty((parts,) + tuple(shape), dtype=np.float32 if dtype == "f32" else np.uint16)

    def job(p):
        _normal(seed, tag, shape, sigma, dtype, part=p, out=out[p])

    if threads > 1 and parts > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(job, range(parts)))
    else:
        for p in range(parts):
            job(p)
    return out


def expert_bias(w: Workload) -> np.ndarray:
    if w.bias:
        return np.asarray(w.bias, dtype=np.float32)
    if w.zipf_s > 0:
        return np.asarray([(e + 1.0) ** (-w.zipf_s) for e in range(w.E)], dtype=np.float32)
    return np.zeros(w.E, dtype=np.float32)


def make_router_inputs(w: Workload) -> dict:
    """Only the routing inputs (cheap even at full size)."""
    out = {}
    if w.mode == "moe":
        lg = _rng(w.seed, "logits").standard_normal((w.T, w.E), dtype=np.float32)
        out["logits"] = (lg + expert_bias(w)[None, :]).astype(np.float32)
    elif w.mode == "mod":
        assert w.B * w.S == w.T
        out["scores"] = _rng(w.seed, "scores").standard_normal((w.B, w.S), dtype=np.float32)
    elif w.mode == "early_exit":
        out["exit_layer"] = _rng(w.seed, "exit").geometric(w.exit_p, size=w.T).astype(np.int32)
    else:
        raise ValueError(w.mode)
    return out


def make_inputs(w: Workload, threads: int = 8) -> dict:
    """All inputs of one workload as numpy arrays.  Floating tensors are
    float32 when w.dtype == "f32" and uint16 bf16 bit patterns otherwise.
    Weights have a leading [layers, E] (early_exit) or [E] dimension."""
    out = make_router_inputs(w)
    out["x"] = _normal(w.seed, "x", (w.T, w.H), 1.0, w.dtype)
    out["dout"] = _normal(w.seed, "dout", (w.T, w.H), 1.0, w.dtype)
    parts = w.E * w.layers
    lead = (w.layers, w.E) if w.mode == "early_exit" else (w.E,)
    for tag, shape in (("Wg", (w.F, w.H)), ("Wu", (w.F, w.H)), ("Wd", (w.H, w.F))):
        a = _per_part(w.seed, tag, parts, shape, 0.02, w.dtype, threads)
        out[tag] = a.reshape(lead + shape)
    return out


def as_f32(a: np.ndarray) -> np.ndarray:
    """The exact fp32 value of a generated tensor, whichever storage it has."""
    return widen_bf16(a) if a.dtype == np.uint16 else a
