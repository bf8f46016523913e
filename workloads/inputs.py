"""Seeded synthetic inputs for the workload subgraphs.

Every tensor is drawn on the host in float64 from its own counter-based stream
``numpy.random.default_rng([seed, config_index, tensor_index])`` and then
rounded (round-to-nearest-even) to its storage dtype.  Nothing here evaluates
any op of a subgraph.

Storage representation handed to both the oracle and the GPU binding:
  f32 -> numpy float32, f16 -> numpy float16, bf16 -> numpy uint16 bit patterns,
  i32 -> numpy int32.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from .graphs import GraphSpec

CONFIG_INDEX = {"pattern": 11, "rmsnorm": 10, "softmax_backward": 8, "layernorm_backward": 9, "softmax": 1, "add_bias_layernorm": 2, "attention_scores": 3,
                "bias_gelu_dbias": 4, "transpose_chain": 5, "transpose": 6, "bias_gelu": 7}


def f64_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float64 -> float32 -> bfloat16 (nearest-even), return uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def quantise(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    if dtype == "f16":
        return np.ascontiguousarray(a, dtype=np.float64).astype(np.float16)
    if dtype == "bf16":
        return f64_to_bf16_bits(a)
    if dtype == "i32":
        return np.ascontiguousarray(a).astype(np.int32)
    raise ValueError(dtype)


def _kind(graph: GraphSpec) -> str:
    for k in sorted(CONFIG_INDEX, key=len, reverse=True):
        if graph.name.startswith(k + "_"):
            return k
    raise ValueError(f"unknown workload kind: {graph.name}")


def _rng(seed: int, cfg: int, tensor: int) -> np.random.Generator:
    return np.random.default_rng([seed, cfg, tensor])


def valid_lengths(batch: int, k_len: int, seed: int = 0) -> np.ndarray:
    """Per-batch valid key length, uniform integer in [min(16,k_len), k_len] inclusive."""
    lo = min(16, k_len)
    return _rng(seed, CONFIG_INDEX["attention_scores"], 100).integers(lo, k_len + 1, size=batch)


def make_inputs(graph: GraphSpec, seed: int = 0) -> Dict[str, np.ndarray]:
    """Storage-dtype inputs of `graph`, keyed by tensor name.

    Distributions (second parameter of N is the standard deviation):
      softmax            x ~ N(0,1)
      add_bias_layernorm x,res ~ N(0,1); bias,beta ~ N(0,0.02); gamma ~ 1+N(0,0.02)
      attention_scores   scores ~ N(0,3); mask 0 / -10000 from per-batch valid length
      bias_gelu(_dbias)  x,grad ~ N(0,1); bias ~ N(0,0.02)
      transpose_chain    x ~ U(-1,1); scale ~ U(0.5,1.5)
      transpose          element i holds the bit pattern of the integer i (index encoding)
      softmax_backward   y ~ Dirichlet(1,..,1) per row (positive, rows sum to 1); dy ~ N(0,1)
      rmsnorm            x ~ N(0,1); gamma ~ 1+N(0,0.02)
      layernorm_backward h, dy ~ N(0,1); gamma ~ 1+N(0,0.02); mu ~ N(0,0.05); rstd ~ U(0.8,1.2)
      pattern (any other pattern or multi-pattern graph) by tensor name (a segment prefix s<k>_ is ignored):
                         g* ~ 1+N(0,0.02); r* ~ U(0.8,1.2); mu* ~ N(0,0.05); bias*, beta* ~ N(0,0.02);
                         mask* 0 / -10000 from per-batch valid length; everything else ~ N(0,1)
    """
    kind = _kind(graph)
    cfg = CONFIG_INDEX[kind]
    out: Dict[str, np.ndarray] = {}
    for ti, t in enumerate(graph.inputs):
        g = _rng(seed, cfg, ti)
        n = key = t.name
        if kind == "softmax":
            a = g.standard_normal(t.dims)
        elif kind == "add_bias_layernorm":
            if n in ("x", "res"):
                a = g.standard_normal(t.dims)
            elif n == "gamma":
                a = 1.0 + 0.02 * g.standard_normal(t.dims)
            else:
                a = 0.02 * g.standard_normal(t.dims)
        elif kind == "attention_scores":
            if n == "scores":
                a = 3.0 * g.standard_normal(t.dims)
            else:
                batch, k_len = t.dims[0], t.dims[-1]
                lens = valid_lengths(batch, k_len, seed)
                a = np.where(np.arange(k_len)[None, :] < lens[:, None], 0.0, -10000.0)
                a = a.reshape(t.dims)
        elif kind in ("bias_gelu_dbias", "bias_gelu"):
            a = g.standard_normal(t.dims) if n in ("x", "grad") else 0.02 * g.standard_normal(t.dims)
        elif kind == "rmsnorm":
            a = g.standard_normal(t.dims) if n == "x" else 1.0 + 0.02 * g.standard_normal(t.dims)
        elif kind == "softmax_backward":
            a = g.dirichlet(np.ones(t.dims[-1]), size=t.dims[:-1]) if n == "y" else g.standard_normal(t.dims)
        elif kind == "layernorm_backward":
            if n in ("h", "dy"):
                a = g.standard_normal(t.dims)
            elif n == "gamma":
                a = 1.0 + 0.02 * g.standard_normal(t.dims)
            elif n == "mu":
                a = 0.05 * g.standard_normal(t.dims)
            else:
                a = g.uniform(0.8, 1.2, t.dims)
        elif kind == "pattern":
            base = n.split("_", 1)[1] if n[0] == "s" and "_" in n and n[1:n.index("_")].isdigit() else n   # segment prefix s<k>_
            if base.startswith("mask"):
                batch, k_len = t.dims[0], t.dims[-1]
                lens = valid_lengths(batch, k_len, seed)
                a = np.where(np.arange(k_len)[None, :] < lens[:, None], 0.0, -10000.0).reshape(t.dims)
                out[key] = quantise(a, t.dtype)
                continue
            n = base
            if n.startswith("g"):
                a = 1.0 + 0.02 * g.standard_normal(t.dims)
            elif n.startswith("r") and n != "res":
                a = g.uniform(0.8, 1.2, t.dims)
            elif n.startswith("mu"):
                a = 0.05 * g.standard_normal(t.dims)
            elif n.startswith(("bias", "beta")):
                a = 0.02 * g.standard_normal(t.dims)
            else:
                a = g.standard_normal(t.dims)
        elif kind == "transpose_chain":
            a = g.uniform(-1.0, 1.0, t.dims) if n == "x" else g.uniform(0.5, 1.5, t.dims)
        elif kind == "transpose":
            count = int(np.prod(t.dims)) if len(t.dims) else 1
            idx = np.arange(count, dtype=np.uint32).reshape(t.dims)
            if t.dtype == "f32":
                out[n] = idx.view(np.float32)
            elif t.dtype == "i32":
                out[n] = idx.view(np.int32)
            elif t.dtype == "f16":
                out[n] = idx.astype(np.uint16).view(np.float16)
            else:
                out[n] = idx.astype(np.uint16)
            continue
        else:  # pragma: no cover
            raise ValueError(kind)
        out[key] = quantise(a, t.dtype)
    return out
