"""CPU oracle for stitched memory-intensive subgraphs.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's `cpu_baseline` leg may
import this module; the product (the HIP library and its binding) never does.

What it computes.  A fused kernel must give the same result as running the ops
of the fusion pattern one after another (Section 7.2 of the paper: results are
unchanged by fusion).  So the oracle is that plain definition: every op of the
subgraph is evaluated on its own, in topological (list) order, each
intermediate materialised as a float64 numpy array.  No blocking, fusion or
reordering.  Op vocabulary = the memory-intensive ops of Section 1 / 3.1 / 4
(elementwise light and expensive, reduction, broadcast, transpose).

Readings of points the paper leaves open (it states no numerics at all):
  * inputs are the already-quantised storage tensors, converted exactly to f64;
  * reductions keep the reduced axis (extent 1); binary ops broadcast numpy-style;
  * reduce_mean divides the sum by the axis extent; variance in the LayerNorm
    subgraph is therefore the population variance of squared deviations;
  * tanh-GELU: gelu(z) = z/2 * (1 + tanh(u)), u = sqrt(2/pi) * (z + 0.044715 z^3),
    and gelu_tanh_grad is its derivative with respect to z;
  * log is the natural logarithm, sigmoid(x) = 1 / (1 + exp(-x)), relu(x) = max(x, 0);
  * `convert` rounds to the target dtype (nearest-even) when other ops consume
    it; when it produces a subgraph output the un-rounded float64 value is
    reported unless `round_outputs=True`, so the comparison tolerance, not the
    oracle, absorbs storage rounding.

Pins (tests/test_oracle_pins.py): closed forms, invariants, brute force in
pure Python, hand-computed values under tests/golden/.  No function here is
"parity unpinned".
"""
from __future__ import annotations

import math
from typing import Dict, Mapping

import numpy as np

SQRT_2_OVER_PI = math.sqrt(2.0 / math.pi)
GELU_C = 0.044715


# --------------------------------------------------------------------------
# storage dtype <-> float64
# --------------------------------------------------------------------------
def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a storage tensor to float64."""
    if dtype == "bf16":
        bits = np.asarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    if dtype == "f16":
        return np.asarray(a, dtype=np.float16).astype(np.float64)
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "i32":
        return np.asarray(a, dtype=np.int32).astype(np.float64)
    raise ValueError(dtype)


def round_to(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to `dtype` (nearest, ties to even), result back in float64."""
    a = np.asarray(a, dtype=np.float64)
    if dtype == "f32":
        return a.astype(np.float32).astype(np.float64)
    if dtype == "f16":
        return a.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        # Exact: scale so the bf16 grid (8 significant bits) is the integers, round half to even.
        out = np.zeros_like(a)
        nz = (a != 0) & np.isfinite(a)
        m, e = np.frexp(a[nz])                 # a = m * 2**e, 0.5 <= |m| < 1
        e = np.maximum(e, -125)                # below the normal range the grid spacing is fixed at 2**-133
        q = np.rint(np.ldexp(a[nz], 8 - e))    # np.rint rounds half to even
        out[nz] = np.ldexp(q, e - 8)
        out[~nz] = a[~nz]
        return out
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# one function per op
# --------------------------------------------------------------------------
def op_add(a, b):
    return a + b


def op_sub(a, b):
    return a - b


def op_mul(a, b):
    return a * b


def op_div(a, b):
    return a / b


def op_max(a, b):
    return np.maximum(a, b)


def op_scale(a, value):
    return a * float(value)


def op_add_scalar(a, value):
    return a + float(value)


def op_square(a):
    return a * a


def op_exp(a):
    return np.exp(a)


def op_rsqrt(a):
    return 1.0 / np.sqrt(a)


def op_tanh(a):
    return np.tanh(a)


def op_gelu_tanh(z):
    u = SQRT_2_OVER_PI * (z + GELU_C * z * z * z)
    return 0.5 * z * (1.0 + np.tanh(u))


def op_gelu_tanh_grad(z):
    u = SQRT_2_OVER_PI * (z + GELU_C * z * z * z)
    t = np.tanh(u)
    du = SQRT_2_OVER_PI * (1.0 + 3.0 * GELU_C * z * z)
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * du


def op_log(a):
    return np.log(a)


def op_sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def op_relu(a):
    return np.maximum(a, 0.0)


def op_abs(a):
    return np.abs(a)


def op_sqrt(a):
    return np.sqrt(a)


def op_broadcast(a, dims):
    return np.broadcast_to(a, tuple(dims)).copy()


def op_reduce_sum(a, axis):
    return np.sum(a, axis=axis, keepdims=True)


def op_reduce_max(a, axis):
    return np.max(a, axis=axis, keepdims=True)


def op_reduce_mean(a, axis):
    return np.sum(a, axis=axis, keepdims=True) / a.shape[axis]


def op_transpose(a, perm):
    return np.ascontiguousarray(np.transpose(a, tuple(perm)))


def op_convert(a, dtype):
    return round_to(a, dtype)


_BINARY = {"add": op_add, "sub": op_sub, "mul": op_mul, "div": op_div, "max": op_max}
_UNARY = {"square": op_square, "exp": op_exp, "rsqrt": op_rsqrt, "tanh": op_tanh,
          "gelu_tanh": op_gelu_tanh, "gelu_tanh_grad": op_gelu_tanh_grad,
          "log": op_log, "sigmoid": op_sigmoid, "relu": op_relu, "abs": op_abs, "sqrt": op_sqrt}


def evaluate(graph, inputs: Mapping[str, np.ndarray], round_outputs: bool = False,
             keep_all: bool = False, stored: Mapping[str, np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Evaluate `graph` op by op in float64.

    graph   : object with .inputs (name,dtype,dims), .ops (out,opcode,inputs,attr), .outputs
    inputs  : storage-dtype arrays keyed by input name
    stored  : {name of a `convert` result that is a graph output: float64 array of the values some implementation
              stored for it}.  The ops that read such a result then read the stored values instead of the oracle's
              own rounding, so everything downstream is the exact function of what was stored (an upstream value near
              a rounding tie may legitimately round either way; the choice must not be charged to what is computed
              from it).  The value reported for the `convert` result itself stays the oracle's own.
    returns : {output name: float64 array}; with keep_all every intermediate too.
    """
    env: Dict[str, np.ndarray] = {}
    pre_convert: Dict[str, np.ndarray] = {}
    own: Dict[str, np.ndarray] = {}       # the oracle's own rounding where `stored` replaced it
    for t in graph.inputs:
        a = to_f64(inputs[t.name], t.dtype)
        if tuple(a.shape) != tuple(t.dims):
            raise ValueError(f"input {t.name}: shape {a.shape} != {t.dims}")
        env[t.name] = a
    for op in graph.ops:
        args = [env[n] for n in op.inputs]
        code = op.opcode
        if code in _BINARY:
            r = _BINARY[code](args[0], args[1])
        elif code in _UNARY:
            r = _UNARY[code](args[0])
        elif code == "scale":
            r = op_scale(args[0], op.attr["value"])
        elif code == "add_scalar":
            r = op_add_scalar(args[0], op.attr["value"])
        elif code == "broadcast":
            r = op_broadcast(args[0], op.attr["dims"])
        elif code == "reduce_sum":
            r = op_reduce_sum(args[0], op.attr["axis"])
        elif code == "reduce_max":
            r = op_reduce_max(args[0], op.attr["axis"])
        elif code == "reduce_mean":
            r = op_reduce_mean(args[0], op.attr["axis"])
        elif code == "transpose":
            r = op_transpose(args[0], op.attr["perm"])
        elif code == "convert":
            pre_convert[op.out] = args[0]
            r = op_convert(args[0], op.attr["dtype"])
        else:
            raise ValueError(f"unknown opcode {code}")
        env[op.out] = np.asarray(r, dtype=np.float64)
        if stored is not None and op.out in stored:
            if code != "convert":
                raise ValueError(f"stored value given for {op.out}, which is not the result of a convert")
            own[op.out] = env[op.out]
            env[op.out] = np.asarray(stored[op.out], dtype=np.float64).reshape(env[op.out].shape)
    if keep_all:
        return env
    out: Dict[str, np.ndarray] = {}
    for name, dtype in graph.outputs:
        if round_outputs:
            out[name] = round_to(own.get(name, env[name]), dtype)
        else:
            out[name] = pre_convert.get(name, env[name])
    return out


# --------------------------------------------------------------------------
# comparison metric used by every parity test
# --------------------------------------------------------------------------
def max_rel_err(got: np.ndarray, ref: np.ndarray, floor: float = 0.0) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, floor), with 0/0 := 0."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(got - ref)
    den = np.maximum(np.abs(ref), floor)
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.where(num == 0.0, 0.0, num / den)
    return float(np.max(q)) if q.size else 0.0


def rms(a: np.ndarray) -> float:
    a = np.asarray(a, dtype=np.float64)
    return float(np.sqrt(np.mean(a * a))) if a.size else 0.0
