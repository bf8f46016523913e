"""Subgraph descriptors for the synthetic memory-intensive workloads.

A descriptor is *data*: named tensors, an ordered list of ops (opcode, operand
names, attributes) and the tensors the subgraph hands back.  It carries no
arithmetic; the CPU oracle interprets it one op at a time in float64 and the
GPU binding replays it through the C ABI.  It plays the role of the paper's
"fusion pattern" P_i = (V_i, E_i), a subgraph of memory-intensive ops
(Section 5.1), which is the input of the code generator (Section 4).

Shape conventions
-----------------
* Binary ops broadcast numpy-style: ranks are right-aligned and a dimension of
  extent 1 stretches.
* Reductions keep the reduced axis with extent 1.
* Every op result is a float32 tensor unless the op is ``convert``.
* ``outputs`` lists (tensor name, storage dtype).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

DTYPES = ("f32", "f16", "bf16", "i32")
DTYPE_BYTES = {"f32": 4, "f16": 2, "bf16": 2, "i32": 4}

# opcode -> number of tensor operands
OPCODES = {
    "add": 2, "sub": 2, "mul": 2, "div": 2, "max": 2,
    "scale": 1, "add_scalar": 1,
    "square": 1, "exp": 1, "rsqrt": 1, "tanh": 1,
    "gelu_tanh": 1, "gelu_tanh_grad": 1, "log": 1, "sigmoid": 1, "relu": 1, "abs": 1, "sqrt": 1,
    "broadcast": 1,
    "reduce_sum": 1, "reduce_max": 1, "reduce_mean": 1,
    "transpose": 1, "convert": 1,
}


@dataclass(frozen=True)
class TensorSpec:
    name: str
    dtype: str
    dims: Tuple[int, ...]


@dataclass(frozen=True)
class OpSpec:
    out: str
    opcode: str
    inputs: Tuple[str, ...]
    attr: Dict = field(default_factory=dict)


@dataclass
class GraphSpec:
    name: str
    inputs: List[TensorSpec]
    ops: List[OpSpec]
    outputs: List[Tuple[str, str]]
    # (output name, input name): the input is computed outside the graph (by a matrix product, say) from that output
    external: List[Tuple[str, str]] = field(default_factory=list)

    def input_names(self) -> List[str]:
        return [t.name for t in self.inputs]


def _op(out: str, opcode: str, *inputs: str, **attr) -> OpSpec:
    assert opcode in OPCODES and len(inputs) == OPCODES[opcode], (opcode, inputs)
    return OpSpec(out, opcode, tuple(inputs), dict(attr))


def _softmax_ops(src: str, axis: int, prefix: str = "") -> List[OpSpec]:
    p = prefix
    return [
        _op(p + "m", "reduce_max", src, axis=axis),
        _op(p + "s", "sub", src, p + "m"),
        _op(p + "e", "exp", p + "s"),
        _op(p + "z", "reduce_sum", p + "e", axis=axis),
        _op(p + "y", "div", p + "e", p + "z"),
    ]


def softmax_graph(rows: int, cols: int, dtype: str = "f32") -> GraphSpec:
    """Row softmax: row max, subtract, exp, row sum, divide (5 ops)."""
    return GraphSpec(
        name=f"softmax_{dtype}_{rows}x{cols}",
        inputs=[TensorSpec("x", dtype, (rows, cols))],
        ops=_softmax_ops("x", 1),
        outputs=[("y", dtype)],
    )


def add_bias_layernorm_graph(rows: int, cols: int, eps: float = 1e-5,
                             in_dtype: str = "f32", out_dtype: str = "bf16") -> GraphSpec:
    """Residual add + bias + LayerNorm (12 ops, the last one the storage convert).

    Population variance, two-pass (mean of squared deviations), eps inside the
    square root; two row reductions and one expensive op on the [rows,1] tensor.
    """
    ops = [
        _op("h0", "add", "x", "res"),
        _op("h", "add", "h0", "bias"),
        _op("mu", "reduce_mean", "h", axis=1),
        _op("c", "sub", "h", "mu"),
        _op("q", "square", "c"),
        _op("v", "reduce_mean", "q", axis=1),
        _op("ve", "add_scalar", "v", value=float(eps)),
        _op("r", "rsqrt", "ve"),
        _op("n", "mul", "c", "r"),
        _op("g", "mul", "n", "gamma"),
        _op("o", "add", "g", "beta"),
        _op("out", "convert", "o", dtype=out_dtype),
    ]
    return GraphSpec(
        name=f"add_bias_layernorm_{in_dtype}_{rows}x{cols}",
        inputs=[
            TensorSpec("x", in_dtype, (rows, cols)),
            TensorSpec("res", in_dtype, (rows, cols)),
            TensorSpec("bias", in_dtype, (cols,)),
            TensorSpec("gamma", in_dtype, (cols,)),
            TensorSpec("beta", in_dtype, (cols,)),
        ],
        ops=ops,
        outputs=[("out", out_dtype)],
    )


def attention_scores_graph(batch: int, heads: int, q_len: int, k_len: int,
                           scale: float = 0.125, dtype: str = "f16") -> GraphSpec:
    """Scale, additive key mask [batch,1,1,k_len], softmax over the last axis (7 ops)."""
    ops = [
        _op("t", "scale", "scores", value=float(scale)),
        _op("a", "add", "t", "mask"),
    ] + _softmax_ops("a", 3)
    return GraphSpec(
        name=f"attention_scores_{dtype}_{batch}x{heads}x{q_len}x{k_len}",
        inputs=[
            TensorSpec("scores", dtype, (batch, heads, q_len, k_len)),
            TensorSpec("mask", dtype, (batch, 1, 1, k_len)),
        ],
        ops=ops,
        outputs=[("y", dtype)],
    )


def bias_gelu_dbias_graph(rows: int, cols: int, dtype: str = "bf16") -> GraphSpec:
    """Bias + tanh-GELU forward packed with the bias-gradient column sum (5 ops)."""
    ops = [
        _op("z", "add", "x", "bias"),
        _op("y", "gelu_tanh", "z"),
        _op("d", "gelu_tanh_grad", "z"),
        _op("p", "mul", "grad", "d"),
        _op("dbias", "reduce_sum", "p", axis=0),
    ]
    return GraphSpec(
        name=f"bias_gelu_dbias_{dtype}_{rows}x{cols}",
        inputs=[
            TensorSpec("x", dtype, (rows, cols)),
            TensorSpec("bias", dtype, (cols,)),
            TensorSpec("grad", dtype, (rows, cols)),
        ],
        ops=ops,
        outputs=[("y", dtype), ("dbias", "f32")],
    )


def transpose_chain_graph(batch: int, seq: int, heads: int, dim: int,
                          eps: float = 1e-6, dtype: str = "f32") -> GraphSpec:
    """[B,S,H,D] -> [B,H,S,D], per-head scale, L2-normalise the last axis (7 ops)."""
    ops = [
        _op("t", "transpose", "x", perm=(0, 2, 1, 3)),
        _op("u", "mul", "t", "scale"),
        _op("q", "square", "u"),
        _op("ss", "reduce_sum", "q", axis=3),
        _op("e", "add_scalar", "ss", value=float(eps)),
        _op("r", "rsqrt", "e"),
        _op("out", "mul", "u", "r"),
    ]
    return GraphSpec(
        name=f"transpose_chain_{dtype}_{batch}x{seq}x{heads}x{dim}",
        inputs=[
            TensorSpec("x", dtype, (batch, seq, heads, dim)),
            TensorSpec("scale", dtype, (heads, 1, 1)),
        ],
        ops=ops,
        outputs=[("out", dtype)],
    )


def transpose_graph(dims: Sequence[int], perm: Sequence[int], dtype: str = "f32") -> GraphSpec:
    """A single transpose op (moves raw bits; used for the bit-exact checks)."""
    return GraphSpec(
        name=f"transpose_{dtype}_{'x'.join(map(str, dims))}_p{''.join(map(str, perm))}",
        inputs=[TensorSpec("x", dtype, tuple(int(d) for d in dims))],
        ops=[_op("t", "transpose", "x", perm=tuple(int(p) for p in perm))],
        outputs=[("t", dtype)],
    )


def bias_gelu_graph(rows: int, cols: int, dtype: str = "bf16") -> GraphSpec:
    """Bias + tanh-GELU only: a pure elementwise chain (thread composition)."""
    return GraphSpec(
        name=f"bias_gelu_{dtype}_{rows}x{cols}",
        inputs=[TensorSpec("x", dtype, (rows, cols)), TensorSpec("bias", dtype, (cols,))],
        ops=[_op("z", "add", "x", "bias"), _op("y", "gelu_tanh", "z")],
        outputs=[("y", dtype)],
    )


def softmax_backward_graph(rows: int, cols: int, dtype: str = "f32") -> GraphSpec:
    """Row softmax backward: dx = y * (dy - sum_j y_j dy_j)  (4 ops, one row reduction)."""
    ops = [
        _op("p", "mul", "y", "dy"),
        _op("s", "reduce_sum", "p", axis=1),
        _op("d", "sub", "dy", "s"),
        _op("dx", "mul", "y", "d"),
    ]
    return GraphSpec(
        name=f"softmax_backward_{dtype}_{rows}x{cols}",
        inputs=[TensorSpec("y", dtype, (rows, cols)), TensorSpec("dy", dtype, (rows, cols))],
        ops=ops,
        outputs=[("dx", dtype)],
    )


def rmsnorm_graph(rows: int, cols: int, eps: float = 1e-6, dtype: str = "bf16") -> GraphSpec:
    """RMS normalisation: x * rsqrt(mean(x^2) + eps) * gamma  (6 ops, one row reduction)."""
    ops = [
        _op("q", "square", "x"),
        _op("v", "reduce_mean", "q", axis=1),
        _op("ve", "add_scalar", "v", value=float(eps)),
        _op("r", "rsqrt", "ve"),
        _op("n", "mul", "x", "r"),
        _op("out", "mul", "n", "gamma"),
    ]
    return GraphSpec(
        name=f"rmsnorm_{dtype}_{rows}x{cols}",
        inputs=[TensorSpec("x", dtype, (rows, cols)), TensorSpec("gamma", dtype, (cols,))],
        ops=ops,
        outputs=[("out", dtype)],
    )


def layernorm_backward_graph(rows: int, cols: int, dtype: str = "f32") -> GraphSpec:
    """LayerNorm backward from saved per-row mean and reciprocal standard deviation (13 ops):
    two row reductions for dx, two column reductions for dgamma and dbeta."""
    ops = [
        _op("c", "sub", "h", "mu"),
        _op("xh", "mul", "c", "rstd"),
        _op("g", "mul", "dy", "gamma"),
        _op("m1", "reduce_mean", "g", axis=1),
        _op("gx", "mul", "g", "xh"),
        _op("m2", "reduce_mean", "gx", axis=1),
        _op("t1", "sub", "g", "m1"),
        _op("t2", "mul", "xh", "m2"),
        _op("t3", "sub", "t1", "t2"),
        _op("dx", "mul", "t3", "rstd"),
        _op("dyx", "mul", "dy", "xh"),
        _op("dgamma", "reduce_sum", "dyx", axis=0),
        _op("dbeta", "reduce_sum", "dy", axis=0),
    ]
    return GraphSpec(
        name=f"layernorm_backward_{dtype}_{rows}x{cols}",
        inputs=[
            TensorSpec("h", dtype, (rows, cols)), TensorSpec("dy", dtype, (rows, cols)),
            TensorSpec("gamma", dtype, (cols,)),
            TensorSpec("mu", "f32", (rows, 1)), TensorSpec("rstd", "f32", (rows, 1)),
        ],
        ops=ops,
        outputs=[("dx", dtype), ("dgamma", "f32"), ("dbeta", "f32")],
    )


# The five configurations the build is measured on, at their full sizes, and a
# small sibling of each that still spans several tiles and a ragged tail.
# Backward patterns measured next to them (same transformer-block shapes).
NEXT_CONFIGS = {
    "N1": lambda: softmax_backward_graph(32 * 12 * 128, 128, "f16"),
    "N2": lambda: layernorm_backward_graph(8192, 768, "f32"),
    "N3": lambda: transpose_graph((64, 512, 12, 64), (0, 2, 3, 1), "f32"),   # innermost axis moves: [B,S,H,D] -> [B,H,D,S]
    "N4": lambda: transpose_graph((64, 512, 12, 64), (0, 2, 3, 1), "bf16"),
    "N5": lambda: rmsnorm_graph(8192, 4096, dtype="bf16"),
    "N6": lambda: layernorm_stats_graph(8192, 768),                          # C2 that also saves mean and rstd for backward
}

# ---- row-local patterns no hand-written kernel family covers (served by the row-program compiler: generated kernel or interpreter) ----
def layernorm_stats_graph(rows: int, cols: int, eps: float = 1e-5, in_dtype: str = "f32", out_dtype: str = "bf16",
                          with_variance: bool = False) -> GraphSpec:
    """Residual add + bias + LayerNorm that also hands out the per-row mean and reciprocal standard
    deviation, as a training forward pass does (three outputs, two of them [rows,1]).  with_variance adds the
    row variance as a fourth output, which no hand-written kernel provides."""
    base = add_bias_layernorm_graph(rows, cols, eps, in_dtype, out_dtype)
    outputs = [("out", out_dtype), ("mu", "f32"), ("r", "f32")] + ([("v", "f32")] if with_variance else [])
    return GraphSpec(name=f"pattern_layernorm_stats_{in_dtype}_{rows}x{cols}", inputs=base.inputs, ops=base.ops, outputs=outputs)


def silu_gate_graph(rows: int, cols: int, dtype: str = "bf16") -> GraphSpec:
    """Gated SiLU: out = a * sigmoid(a) * b with sigmoid spelt as 1 / (1 + exp(-a))  (6 ops, no reduction)."""
    ops = [
        _op("n", "scale", "a", value=-1.0),
        _op("e", "exp", "n"),
        _op("d", "add_scalar", "e", value=1.0),
        _op("s", "div", "a", "d"),
        _op("out", "mul", "s", "b"),
    ]
    return GraphSpec(name=f"pattern_silu_gate_{dtype}_{rows}x{cols}",
                     inputs=[TensorSpec("a", dtype, (rows, cols)), TensorSpec("b", dtype, (rows, cols))],
                     ops=ops, outputs=[("out", dtype)])


def log_softmax_graph(rows: int, cols: int, dtype: str = "f32") -> GraphSpec:
    """Row log-softmax: y = (x - max) - log(sum exp(x - max))  (6 ops, two row reductions)."""
    ops = [_op("m", "reduce_max", "x", axis=1), _op("c", "sub", "x", "m"), _op("e", "exp", "c"),
           _op("s", "reduce_sum", "e", axis=1), _op("l", "log", "s"), _op("y", "sub", "c", "l")]
    return GraphSpec(name=f"pattern_log_softmax_{dtype}_{rows}x{cols}", inputs=[TensorSpec("x", dtype, (rows, cols))],
                     ops=ops, outputs=[("y", dtype)])


def sigmoid_gate_graph(rows: int, cols: int, dtype: str = "bf16") -> GraphSpec:
    """Gated linear unit with a rectified side branch: out = a * sigmoid(b + bias) + relu(a)  (5 ops)."""
    ops = [_op("z", "add", "b", "bias"), _op("g", "sigmoid", "z"), _op("p", "mul", "a", "g"), _op("r", "relu", "a"),
           _op("out", "add", "p", "r")]
    return GraphSpec(name=f"pattern_sigmoid_gate_{dtype}_{rows}x{cols}",
                     inputs=[TensorSpec("a", dtype, (rows, cols)), TensorSpec("b", dtype, (rows, cols)), TensorSpec("bias", dtype, (cols,))],
                     ops=ops, outputs=[("out", dtype)])


def l1_l2_scale_graph(rows: int, cols: int, dtype: str = "f32", eps: float = 1e-6) -> GraphSpec:
    """Rows scaled by their L2 norm, and their L1 norms: out = x / sqrt(sum x^2 + eps), l1 = sum |x|  (7 ops)."""
    ops = [_op("q", "square", "x"), _op("ss", "reduce_sum", "q", axis=1), _op("e", "add_scalar", "ss", value=float(eps)),
           _op("n", "sqrt", "e"), _op("out", "div", "x", "n"), _op("a", "abs", "x"), _op("l1", "reduce_sum", "a", axis=1)]
    return GraphSpec(name=f"pattern_l1_l2_scale_{dtype}_{rows}x{cols}", inputs=[TensorSpec("x", dtype, (rows, cols))],
                     ops=ops, outputs=[("out", dtype), ("l1", "f32")])


def scaled_softmax_colbias_graph(rows: int, cols: int, dtype: str = "f32") -> GraphSpec:
    """softmax(scale * x + colbias) followed by a per-column gain: a softmax neighbourhood the softmax family
    does not match (column-vector operands on both sides)."""
    ops = [_op("t", "scale", "x", value=0.5), _op("a", "add", "t", "bias")] + _softmax_ops("a", 1) + [_op("out", "mul", "y", "gamma")]
    return GraphSpec(name=f"pattern_softmax_colbias_{dtype}_{rows}x{cols}",
                     inputs=[TensorSpec("x", dtype, (rows, cols)), TensorSpec("bias", dtype, (cols,)), TensorSpec("gamma", dtype, (cols,))],
                     ops=ops, outputs=[("out", dtype)])


def normalize_from_stats_graph(rows: int, cols: int, dtype: str = "f16") -> GraphSpec:
    """(h - mu) * rstd * gamma with saved per-row statistics as inputs, an explicit broadcast op, and the row
    maximum of the result stretched back to [rows, cols] as a second output."""
    ops = [
        _op("mb", "broadcast", "mu", dims=(rows, cols)),
        _op("c", "sub", "h", "mb"),
        _op("n", "mul", "c", "rstd"),
        _op("out", "mul", "n", "gamma"),
        _op("top", "reduce_max", "out", axis=1),
        _op("topb", "broadcast", "top", dims=(rows, cols)),
    ]
    return GraphSpec(name=f"pattern_normalize_from_stats_{dtype}_{rows}x{cols}",
                     inputs=[TensorSpec("h", dtype, (rows, cols)), TensorSpec("gamma", dtype, (cols,)),
                             TensorSpec("mu", "f32", (rows, 1)), TensorSpec("rstd", "f32", (rows, 1))],
                     ops=ops, outputs=[("out", dtype), ("topb", "f32")])


def outer_scale_graph(rows: int, cols: int) -> GraphSpec:
    """out = tanh(gamma[cols] * rstd[rows,1]): a full-shaped result with no full-shaped input."""
    ops = [_op("p", "mul", "gamma", "rstd"), _op("out", "tanh", "p")]
    return GraphSpec(name=f"pattern_outer_scale_f32_{rows}x{cols}",
                     inputs=[TensorSpec("gamma", "f32", (cols,)), TensorSpec("rstd", "f32", (rows, 1))],
                     ops=ops, outputs=[("out", "f32")])


def masked_scores_gate_graph(batch: int, heads: int, q_len: int, k_len: int, dtype: str = "f16") -> GraphSpec:
    """Attention scores with an additive key mask [batch,1,1,k_len], a per-head temperature [heads,1,1] and a
    tanh soft-cap before the softmax: a softmax neighbourhood with two operands stretched along different
    leading axes, which the softmax family does not match."""
    ops = [
        _op("t", "mul", "scores", "temp"),
        _op("cap", "tanh", "t"),
        _op("c30", "scale", "cap", value=30.0),
        _op("a", "add", "c30", "mask"),
    ] + _softmax_ops("a", 3)
    return GraphSpec(name=f"pattern_masked_gate_{dtype}_{batch}x{heads}x{q_len}x{k_len}",
                     inputs=[TensorSpec("scores", dtype, (batch, heads, q_len, k_len)), TensorSpec("mask", dtype, (batch, 1, 1, k_len)),
                             TensorSpec("temp", "f32", (heads, 1, 1))],
                     ops=ops, outputs=[("y", dtype)])


def bias_head_split_graph(batch: int, seq: int, heads: int, dim: int, dtype: str = "bf16") -> GraphSpec:
    """Projection bias, then the head split: x[B,S,H,D] + bias[H,D], stored as [B,H,S,D].  The transpose keeps the
    innermost axis, so a row kernel can fold it into its store."""
    # arithmetic results are float32; a transpose moves values as they are, so the rounding to the storage dtype
    # is an op of its own in front of it
    ops = [_op("z", "add", "x", "bias")]
    if dtype != "f32":
        ops.append(_op("zc", "convert", "z", dtype=dtype))
    ops.append(_op("out", "transpose", ops[-1].out, perm=(0, 2, 1, 3)))
    return GraphSpec(name=f"pattern_bias_head_split_{dtype}_{batch}x{seq}x{heads}x{dim}",
                     inputs=[TensorSpec("x", dtype, (batch, seq, heads, dim)), TensorSpec("bias", dtype, (heads, dim))],
                     ops=ops, outputs=[("out", dtype)])


def head_merge_residual_graph(batch: int, seq: int, heads: int, dim: int, dtype: str = "bf16") -> GraphSpec:
    """Head merge, then a gain per column and a residual: ctx[B,H,S,D] -> [B,S,H,D], times g[D], plus res[B,S,H,D]
    (the transpose is folded into the load of ctx)."""
    ops = [_op("t", "transpose", "ctx", perm=(0, 2, 1, 3)), _op("u", "mul", "t", "g"), _op("out", "add", "u", "res")]
    return GraphSpec(name=f"pattern_head_merge_{dtype}_{batch}x{seq}x{heads}x{dim}",
                     inputs=[TensorSpec("ctx", dtype, (batch, heads, seq, dim)), TensorSpec("g", dtype, (dim,)),
                             TensorSpec("res", dtype, (batch, seq, heads, dim))],
                     ops=ops, outputs=[("out", dtype)])


def transpose_chain_stats_graph(batch: int, seq: int, heads: int, dim: int, eps: float = 1e-6, dtype: str = "f32") -> GraphSpec:
    """The transpose chain ([B,S,H,D] -> [B,H,S,D], per-head scale, L2-normalise the last axis) that also stores the
    row sums of squares: one more output than the hand-written transpose-chain family takes."""
    ops = [
        _op("t", "transpose", "x", perm=(0, 2, 1, 3)),
        _op("u", "mul", "t", "r_scale"),
        _op("q", "square", "u"),
        _op("ss", "reduce_sum", "q", axis=3),
        _op("e", "add_scalar", "ss", value=float(eps)),
        _op("r", "rsqrt", "e"),
        _op("out", "mul", "u", "r"),
    ]
    return GraphSpec(name=f"pattern_tchain_stats_{dtype}_{batch}x{seq}x{heads}x{dim}",
                     inputs=[TensorSpec("x", dtype, (batch, seq, heads, dim)), TensorSpec("r_scale", dtype, (heads, 1, 1))],
                     ops=ops, outputs=[("out", dtype), ("ss", "f32")])


def transposed_softmax_graph(batch: int, q_len: int, heads: int, k_len: int, dtype: str = "f16") -> GraphSpec:
    """Scores laid out [B,S,H,T], wanted as probabilities [B,H,S,T]: transpose, scale, softmax over T."""
    ops = [_op("t", "transpose", "scores", perm=(0, 2, 1, 3)), _op("a", "scale", "t", value=0.125)] + _softmax_ops("a", 3)
    return GraphSpec(name=f"pattern_transposed_softmax_{dtype}_{batch}x{q_len}x{heads}x{k_len}",
                     inputs=[TensorSpec("scores", dtype, (batch, q_len, heads, k_len))], ops=ops, outputs=[("y", dtype)])


def gelu_backward_graph(rows: int, cols: int, dtype: str = "bf16", sum_dtype: str = "f32") -> GraphSpec:
    """Backward of bias + tanh-GELU: dx = g * gelu'(x + bias) and the bias gradient, the column sum of dx (handed out
    as float32, or rounded once to `sum_dtype`)."""
    ops = [_op("z", "add", "x", "bias"), _op("d", "gelu_tanh_grad", "z"), _op("dx", "mul", "g", "d"),
           _op("dbias", "reduce_sum", "dx", axis=0)]
    return GraphSpec(name=f"pattern_gelu_backward_{dtype}_{rows}x{cols}" + ("" if sum_dtype == "f32" else f"_sum_{sum_dtype}"),
                     inputs=[TensorSpec("x", dtype, (rows, cols)), TensorSpec("bias", dtype, (cols,)), TensorSpec("g", dtype, (rows, cols))],
                     ops=ops, outputs=[("dx", dtype), ("dbias", sum_dtype)])


def bias_gradient_chain_graph(dims: Sequence[int], dtype: str = "bf16") -> GraphSpec:
    """Backward of bias + tanh-GELU over activations with several leading axes ([B,S,H] or [B,S,N,H]): dx, and the bias
    gradient as a chain of sums, one leading axis after the other, down to one value per column."""
    dims = tuple(int(d) for d in dims)
    rank = len(dims)
    ops = [_op("z", "add", "x", "bias"), _op("d", "gelu_tanh_grad", "z"), _op("dx", "mul", "g", "d")]
    prev = "dx"
    for ax in range(rank - 1):
        name = "dbias" if ax == rank - 2 else f"s{ax}"
        ops.append(_op(name, "reduce_sum", prev, axis=ax))
        prev = name
    return GraphSpec(name=f"pattern_bias_gradient_chain_{dtype}_{'x'.join(map(str, dims))}",
                     inputs=[TensorSpec("x", dtype, dims), TensorSpec("bias", dtype, dims[-1:]), TensorSpec("g", dtype, dims)],
                     ops=ops, outputs=[("dx", dtype), ("dbias", "f32")])


def layernorm_backward_bias_graph(rows: int, cols: int, dtype: str = "bf16", sum_dtype: str = "f32") -> GraphSpec:
    """LayerNorm backward from saved statistics together with the gradient of the bias that was added in front of the
    LayerNorm: dx (rounded to the storage dtype), dgamma, dbeta and dbias = column sum of the rounded dx.  Two row
    reductions and three column sums in one pattern."""
    ops = [
        _op("c", "sub", "h", "mu"), _op("xh", "mul", "c", "rstd"), _op("g", "mul", "dy", "gamma"),
        _op("m1", "reduce_mean", "g", axis=1), _op("gx", "mul", "g", "xh"), _op("m2", "reduce_mean", "gx", axis=1),
        _op("t1", "sub", "g", "m1"), _op("t2", "mul", "xh", "m2"), _op("t3", "sub", "t1", "t2"), _op("dx", "mul", "t3", "rstd"),
        _op("dxc", "convert", "dx", dtype=dtype), _op("dbias", "reduce_sum", "dxc", axis=0),
        _op("dyx", "mul", "dy", "xh"), _op("dgamma", "reduce_sum", "dyx", axis=0), _op("dbeta", "reduce_sum", "dy", axis=0),
    ]
    return GraphSpec(name=f"pattern_layernorm_backward_bias_{dtype}_{rows}x{cols}",
                     inputs=[TensorSpec("h", dtype, (rows, cols)), TensorSpec("dy", dtype, (rows, cols)), TensorSpec("gamma", dtype, (cols,)),
                             TensorSpec("mu", "f32", (rows, 1)), TensorSpec("rstd", "f32", (rows, 1))],
                     ops=ops, outputs=[("dxc", dtype), ("dbias", sum_dtype), ("dgamma", sum_dtype), ("dbeta", sum_dtype)])


def rmsnorm_backward_graph(rows: int, cols: int, dtype: str = "bf16") -> GraphSpec:
    """Backward of RMSNorm from the saved reciprocal rms: xhat = x * rrms; dgamma = column sum of dy * xhat;
    gy = dy * gamma; dx = (gy - xhat * rowmean(gy * xhat)) * rrms.  A row reduction and a column reduction in one
    pattern."""
    ops = [
        _op("xhat", "mul", "x", "rrms"),
        _op("dyx", "mul", "dy", "xhat"),
        _op("dgamma", "reduce_sum", "dyx", axis=0),
        _op("gy", "mul", "dy", "g"),
        _op("gx", "mul", "gy", "xhat"),
        _op("m", "reduce_mean", "gx", axis=1),
        _op("xm", "mul", "xhat", "m"),
        _op("c", "sub", "gy", "xm"),
        _op("dx", "mul", "c", "rrms"),
    ]
    return GraphSpec(name=f"pattern_rmsnorm_backward_{dtype}_{rows}x{cols}",
                     inputs=[TensorSpec("x", dtype, (rows, cols)), TensorSpec("dy", dtype, (rows, cols)), TensorSpec("g", dtype, (cols,)),
                             TensorSpec("rrms", "f32", (rows, 1))],
                     ops=ops, outputs=[("dx", dtype), ("dgamma", "f32")])


def random_row_pattern(seed: int, rows: int, cols: int, dtype: str = "f32", n_ops: int = 12, column_sums: int = 0,
                       more_ops: bool = False) -> GraphSpec:
    """A random connected pattern of element-wise ops and row reductions over [rows, cols] (descriptor only).
    Domains are kept safe by construction: exp only of tanh, division and rsqrt only of 1 + square.
    column_sums: up to that many full-shaped values of the pattern are also summed over all rows (float32 outputs).
    more_ops: sigmoid, relu, abs, and log / sqrt of 1 + square join the vocabulary."""
    import random
    rnd = random.Random(seed)
    inputs = [TensorSpec("x0", dtype, (rows, cols))]
    kinds = {"x0": "full"}
    for i in range(rnd.randint(0, 2)):
        inputs.append(TensorSpec(f"x{i + 1}", dtype, (rows, cols)))
        kinds[f"x{i + 1}"] = "full"
    for i in range(rnd.randint(0, 2)):
        inputs.append(TensorSpec(f"g{i}", dtype, (cols,)))
        kinds[f"g{i}"] = "col"
    for i in range(rnd.randint(0, 2)):
        inputs.append(TensorSpec(f"r{i}", "f32", (rows, 1)))
        kinds[f"r{i}"] = "rscal"
    ops: List[OpSpec] = []
    names = list(kinds)

    def pick(want=None):
        pool = [n for n in names if want is None or kinds[n] in want]
        recent = pool[-4:]
        return rnd.choice(recent if rnd.random() < 0.6 else pool)

    def add(opcode, *ins, kind, **attr):
        name = f"v{len(ops)}"
        ops.append(_op(name, opcode, *ins, **attr))
        kinds[name] = kind
        names.append(name)
        return name

    def join(ka, kb):
        if ka == kb and ka != "full":
            return ka
        return "full"

    while len(ops) < n_ops:
        r = rnd.random()
        if more_ops and rnd.random() < 0.3:
            a = pick(("full", "rscal"))
            kind = rnd.choice(["sigmoid", "relu", "abs", "log", "sqrt"])
            if kind in ("log", "sqrt"):
                q = add("square", a, kind=kinds[a])
                a = add("add_scalar", q, kind=kinds[a], value=1.0)
            add(kind, a, kind=kinds[a])
            continue
        if r < 0.40:
            a, b = pick(), pick()
            if kinds[a] == "col" and kinds[b] == "col":
                continue
            op = rnd.choice(["add", "sub", "mul", "max"])
            v = add(op, a, b, kind=join(kinds[a], kinds[b]))
            if op == "mul":
                add("tanh", v, kind=kinds[v])                    # keeps magnitudes bounded
        elif r < 0.55:
            a = pick(("full", "rscal"))
            add(rnd.choice(["scale", "add_scalar"]), a, kind=kinds[a], value=rnd.choice([-1.5, 0.25, 0.5, 2.0]))
        elif r < 0.67:
            a = pick(("full", "rscal"))
            t = add("tanh", a, kind=kinds[a])
            add(rnd.choice(["exp", "gelu_tanh", "square"]), t, kind=kinds[a])
        elif r < 0.77:
            a, b = pick(), pick(("full", "rscal"))
            q = add("square", b, kind=kinds[b])
            d = add("add_scalar", q, kind=kinds[b], value=1.0)
            if rnd.random() < 0.5:
                d = add("rsqrt", d, kind=kinds[b])
                add("mul", a, d, kind=join(kinds[a], kinds[b])) if not (kinds[a] == "col" and kinds[b] == "col") else None
            else:
                add("div", a, d, kind=join(kinds[a], kinds[b]))
        else:
            a = pick(("full",))
            add(rnd.choice(["reduce_sum", "reduce_max", "reduce_mean"]), a, kind="rscal", axis=1)
    # outputs: the last full value, plus up to two more values; ops that reach no output are dropped
    fulls = [o.out for o in ops if kinds[o.out] == "full"]
    if not fulls:
        fulls = [add("add", "x0", names[-1], kind="full")]
    outs = [fulls[-1]]
    extra = [o.out for o in ops if kinds[o.out] in ("full", "rscal") and o.out != outs[0]]
    rnd.shuffle(extra)
    outs += extra[:rnd.randint(0, 2)]
    live = set(outs)
    for o in reversed(ops):
        if o.out in live:
            live.update(o.inputs)
    ops = [o for o in ops if o.out in live]
    inputs = [t for t in inputs if t.name in live] or inputs[:1]
    outputs = [(n, dtype if kinds[n] == "full" else "f32") for n in outs]
    if column_sums > 0:
        summed = [o.out for o in ops if kinds[o.out] == "full"]
        rnd.shuffle(summed)
        for i, n in enumerate(sorted(summed[:column_sums], key=lambda n: int(n[1:]))):
            ops.append(_op(f"cs{i}", "reduce_sum", n, axis=0))
            outputs.append((f"cs{i}", "f32"))
    return GraphSpec(name=f"pattern_random{seed}_{dtype}_{rows}x{cols}" + (f"_cs{column_sums}" if column_sums else "") + ("_more" if more_ops else ""),
                     inputs=inputs, ops=ops, outputs=outputs)


# ---- graphs that hold many fusion patterns (input of the fusion explorer) ----
def _layernorm_ops(prefix: str, x: str, res: str, bias: str, gamma: str, beta: str, eps: float, out_dtype: str) -> List[OpSpec]:
    p = prefix
    return [
        _op(p + "h0", "add", x, res), _op(p + "h", "add", p + "h0", bias),
        _op(p + "mu", "reduce_mean", p + "h", axis=1), _op(p + "c", "sub", p + "h", p + "mu"),
        _op(p + "q", "square", p + "c"), _op(p + "v", "reduce_mean", p + "q", axis=1),
        _op(p + "ve", "add_scalar", p + "v", value=float(eps)), _op(p + "r", "rsqrt", p + "ve"),
        _op(p + "n", "mul", p + "c", p + "r"), _op(p + "g", "mul", p + "n", gamma), _op(p + "o", "add", p + "g", beta),
        _op(p + "out", "convert", p + "o", dtype=out_dtype),
    ]


def transformer_block_graph(batch: int = 32, seq: int = 128, heads: int = 12, dim: int = 64, ffn: int = 3072,
                            dtype: str = "bf16", projection_bias: bool = False, matmul_dependences: bool = True) -> GraphSpec:
    """The memory-intensive ops of one transformer encoder block, with the matrix products taken out: their
    results come in as graph inputs.  Head split / merge transposes, scale + mask + softmax, output bias +
    residual + LayerNorm, feed-forward bias + GELU, second bias + residual + LayerNorm that reads the first
    one's stored result (37 ops, 8 patterns by hand).  projection_bias: the query / key / value projections come
    without their biases [H,D], which are added (and the sum rounded to the storage dtype) in front of the head
    split (43 ops, or 46 with the rounding when the storage dtype is not float32).
    matmul_dependences: the graph says which input each matrix product computes from which outputs (scores from the
    split q and k, the context from probabilities and v, ...), so that no pattern spans a matrix product; without
    them every input counts as available from the start."""
    hidden, rows = heads * dim, batch * seq
    t4 = (batch, seq, heads, dim)
    split, bias_inputs = [], []
    for n in ("q", "k", "v"):
        if projection_bias:
            bias_inputs.append(TensorSpec(f"bias_{n}", dtype, (heads, dim)))
            split.append(_op(f"{n}_b", "add", f"{n}_lin", f"bias_{n}"))
            src = f"{n}_b"
            if dtype != "f32":
                split.append(_op(f"{n}_c", "convert", src, dtype=dtype))
                src = f"{n}_c"
            split.append(_op(f"{n}t", "transpose", src, perm=(0, 2, 1, 3)))
        else:
            split.append(_op(f"{n}t", "transpose", f"{n}_lin", perm=(0, 2, 1, 3)))
    inputs = bias_inputs + [
        TensorSpec("q_lin", dtype, t4), TensorSpec("k_lin", dtype, t4), TensorSpec("v_lin", dtype, t4),
        TensorSpec("scores", dtype, (batch, heads, seq, seq)), TensorSpec("mask", dtype, (batch, 1, 1, seq)),
        TensorSpec("ctx", dtype, (batch, heads, seq, dim)),
        TensorSpec("attn_out", dtype, (rows, hidden)), TensorSpec("x", dtype, (rows, hidden)),
        TensorSpec("bias_o", dtype, (hidden,)), TensorSpec("gamma1", dtype, (hidden,)), TensorSpec("beta1", dtype, (hidden,)),
        TensorSpec("ffn1_out", dtype, (rows, ffn)), TensorSpec("bias1", dtype, (ffn,)),
        TensorSpec("ffn2_out", dtype, (rows, hidden)), TensorSpec("bias2", dtype, (hidden,)),
        TensorSpec("gamma2", dtype, (hidden,)), TensorSpec("beta2", dtype, (hidden,)),
    ]
    ops = split + [
        _op("sc", "scale", "scores", value=float(dim) ** -0.5), _op("sa", "add", "sc", "mask"),
    ] + _softmax_ops("sa", 3, prefix="p_") + [
        _op("ctx_t", "transpose", "ctx", perm=(0, 2, 1, 3)),
    ] + _layernorm_ops("l1_", "attn_out", "x", "bias_o", "gamma1", "beta1", 1e-5, dtype) + [
        _op("f_a", "add", "ffn1_out", "bias1"), _op("act", "gelu_tanh", "f_a"),
    ] + _layernorm_ops("l2_", "ffn2_out", "l1_out", "bias2", "gamma2", "beta2", 1e-5, dtype)
    outputs = [("qt", dtype), ("kt", dtype), ("vt", dtype), ("p_y", dtype), ("ctx_t", dtype), ("l1_out", dtype),
               ("act", dtype), ("l2_out", dtype)]
    # the matrix products that were taken out: what each one reads and what it hands back
    external = [("qt", "scores"), ("kt", "scores"), ("p_y", "ctx"), ("vt", "ctx"), ("ctx_t", "attn_out"), ("l1_out", "ffn1_out"),
                ("act", "ffn2_out")] if matmul_dependences else []
    return GraphSpec(name=f"pattern_transformer_block_{'pb_' if projection_bias else ''}{dtype}_b{batch}_s{seq}", inputs=inputs, ops=ops,
                     outputs=outputs, external=external)


def transformer_stack_graph(n_blocks: int, batch: int = 32, seq: int = 128, heads: int = 12, dim: int = 64, ffn: int = 3072,
                            dtype: str = "bf16") -> GraphSpec:
    """`n_blocks` encoder blocks one after the other: a block's residual input is the previous block's output itself
    (an edge of the graph), its q / k / v projections are matrix products of that output (declared)."""
    inputs: List[TensorSpec] = []
    ops: List[OpSpec] = []
    outputs: List[Tuple[str, str]] = []
    external: List[Tuple[str, str]] = []
    prev_out = None
    for b in range(n_blocks):
        blk = transformer_block_graph(batch, seq, heads, dim, ffn, dtype)
        ren = lambda n, b=b: f"b{b}_{n}"
        src = lambda n, b=b, prev=prev_out: prev if (n == "x" and prev is not None) else f"b{b}_{n}"
        inputs += [TensorSpec(ren(t.name), t.dtype, t.dims) for t in blk.inputs if not (t.name == "x" and prev_out is not None)]
        ops += [OpSpec(ren(o.out), o.opcode, tuple(src(i) for i in o.inputs), dict(o.attr)) for o in blk.ops]
        outputs += [(ren(n), d) for n, d in blk.outputs]
        external += [(ren(a), ren(c)) for a, c in blk.external]
        if prev_out is not None:
            external += [(prev_out, ren(n)) for n in ("q_lin", "k_lin", "v_lin")]
        prev_out = ren("l2_out")
    return GraphSpec(name=f"pattern_transformer_stack{n_blocks}_{dtype}_b{batch}_s{seq}", inputs=inputs, ops=ops, outputs=outputs,
                     external=external)


def transformer_block_backward_graph(batch: int = 32, seq: int = 128, heads: int = 12, dim: int = 64, ffn: int = 3072,
                                     dtype: str = "bf16", matmul_dependences: bool = True) -> GraphSpec:
    """The memory-intensive ops of the backward pass through one transformer encoder block, matrix products taken out
    (the gradients they produce come in as graph inputs, the gradients they consume go out as graph outputs):
    LayerNorm 2 backward from saved statistics (dx, dgamma, dbeta) and the bias gradient behind it, bias + GELU
    backward with its bias gradient, the residual sum into LayerNorm 1 backward and its bias gradient, softmax backward
    on the attention probabilities with the score scale, and the head split / merge transposes of the gradients.
    Row reductions, column sums over all rows and transposes side by side (45 ops)."""
    hidden, rows = heads * dim, batch * seq
    t_bshd, t_bhsd = (batch, seq, heads, dim), (batch, heads, seq, dim)

    def ln_backward(p: str, h: str, dy: str, gamma: str, mu: str, rstd: str) -> List[OpSpec]:
        return [
            _op(p + "c", "sub", h, mu), _op(p + "xh", "mul", p + "c", rstd), _op(p + "g", "mul", dy, gamma),
            _op(p + "m1", "reduce_mean", p + "g", axis=1), _op(p + "gx", "mul", p + "g", p + "xh"),
            _op(p + "m2", "reduce_mean", p + "gx", axis=1), _op(p + "t1", "sub", p + "g", p + "m1"),
            _op(p + "t2", "mul", p + "xh", p + "m2"), _op(p + "t3", "sub", p + "t1", p + "t2"),
            _op(p + "dx", "mul", p + "t3", rstd), _op(p + "dxc", "convert", p + "dx", dtype=dtype),
            _op(p + "dyx", "mul", dy, p + "xh"), _op(p + "dgamma", "reduce_sum", p + "dyx", axis=0),
            _op(p + "dbeta", "reduce_sum", dy, axis=0),
        ]

    inputs = [
        TensorSpec("dy2", dtype, (rows, hidden)), TensorSpec("h2", dtype, (rows, hidden)), TensorSpec("gamma2", dtype, (hidden,)),
        TensorSpec("mu2", "f32", (rows, 1)), TensorSpec("rstd2", "f32", (rows, 1)),
        TensorSpec("ffn1_pre", dtype, (rows, ffn)), TensorSpec("bias1", dtype, (ffn,)), TensorSpec("up_act", dtype, (rows, ffn)),
        TensorSpec("up_l1", dtype, (rows, hidden)), TensorSpec("h1", dtype, (rows, hidden)), TensorSpec("gamma1", dtype, (hidden,)),
        TensorSpec("mu1", "f32", (rows, 1)), TensorSpec("rstd1", "f32", (rows, 1)),
        TensorSpec("probs", dtype, (batch, heads, seq, seq)), TensorSpec("up_probs", dtype, (batch, heads, seq, seq)),
        TensorSpec("up_ctx", dtype, t_bshd), TensorSpec("up_q", dtype, t_bhsd), TensorSpec("up_k", dtype, t_bhsd),
        TensorSpec("up_v", dtype, t_bhsd),
    ]
    ops = ln_backward("l2_", "h2", "dy2", "gamma2", "mu2", "rstd2") + [
        _op("dbias2", "reduce_sum", "l2_dxc", axis=0),
        _op("f_z", "add", "ffn1_pre", "bias1"), _op("f_d", "gelu_tanh_grad", "f_z"), _op("f_dx", "mul", "up_act", "f_d"),
        _op("f_dxc", "convert", "f_dx", dtype=dtype), _op("dbias1", "reduce_sum", "f_dxc", axis=0),
        _op("dy1", "add", "l2_dxc", "up_l1"),
    ] + ln_backward("l1_", "h1", "dy1", "gamma1", "mu1", "rstd1") + [
        _op("dbias_o", "reduce_sum", "l1_dxc", axis=0),
        _op("d_ctx", "transpose", "up_ctx", perm=(0, 2, 1, 3)),
        _op("a_p", "mul", "probs", "up_probs"), _op("a_s", "reduce_sum", "a_p", axis=3), _op("a_d", "sub", "up_probs", "a_s"),
        _op("a_ds", "mul", "probs", "a_d"), _op("d_scores", "scale", "a_ds", value=float(dim) ** -0.5),
        _op("d_q", "transpose", "up_q", perm=(0, 2, 1, 3)), _op("d_k", "transpose", "up_k", perm=(0, 2, 1, 3)),
        _op("d_v", "transpose", "up_v", perm=(0, 2, 1, 3)),
    ]
    outputs = [("l2_dxc", dtype), ("l2_dgamma", "f32"), ("l2_dbeta", "f32"), ("dbias2", "f32"), ("f_dxc", dtype), ("dbias1", "f32"),
               ("l1_dxc", dtype), ("l1_dgamma", "f32"), ("l1_dbeta", "f32"), ("dbias_o", "f32"), ("d_ctx", dtype), ("d_scores", dtype),
               ("d_q", dtype), ("d_k", dtype), ("d_v", dtype)]
    # the backward matrix products that were taken out: the gradient each one computes from which gradient
    external = [("l2_dxc", "up_act"), ("f_dxc", "up_l1"), ("l1_dxc", "up_ctx"), ("d_ctx", "up_probs"), ("d_ctx", "up_v"),
                ("d_scores", "up_q"), ("d_scores", "up_k")] if matmul_dependences else []
    return GraphSpec(name=f"pattern_transformer_block_backward_{dtype}_b{batch}_s{seq}", inputs=inputs, ops=ops, outputs=outputs,
                     external=external)


def random_multi_pattern(seed: int, rows: int = 24, cols: int = 32, segments: int = 3, dtype: str = "f32",
                         seg_ops: Tuple[int, int] = (3, 9), column_sums: int = 0, external_links: bool = False) -> GraphSpec:
    """Several random row patterns chained through transposes (each transpose turns the previous segment's
    columns into rows, so no single row kernel can span it) plus an independent side pattern.
    external_links: every other link of the chain is a computation outside the graph instead (the next segment's
    first input is declared as computed from the previous segment's main output)."""
    import random
    rnd = random.Random(1000 + seed)
    inputs: List[TensorSpec] = []
    ops: List[OpSpec] = []
    outputs: List[Tuple[str, str]] = []
    carry = None
    external: List[Tuple[str, str]] = []
    outside_source = None
    r, c = rows, cols
    for s in range(segments):
        seg = random_row_pattern(seed * 17 + s, r, c, dtype, n_ops=rnd.randint(*seg_ops), column_sums=column_sums)
        ren = {t.name: f"s{s}_{t.name}" for t in seg.inputs}
        ren.update({o.out: f"s{s}_{o.out}" for o in seg.ops})
        seg_inputs = list(seg.inputs)
        if outside_source is not None:
            external.append((outside_source, ren[seg_inputs[0].name]))   # this segment's first input comes from outside
            outside_source = None
        if carry is not None:
            ren[seg_inputs[0].name] = carry                      # the first full input is the transposed carry
            seg_inputs = seg_inputs[1:]
        inputs += [TensorSpec(ren[t.name], t.dtype, t.dims) for t in seg_inputs]
        ops += [OpSpec(ren[o.out], o.opcode, tuple(ren[i] for i in o.inputs), dict(o.attr)) for o in seg.ops]
        main = ren[seg.outputs[0][0]]
        for name, dt in seg.outputs[1:]:
            outputs.append((ren[name], dt))
        if s + 1 < segments and external_links and s % 2 == 0:
            outputs.append((main, dtype))          # what the outside computation reads
            outside_source = main
            carry = None
        elif s + 1 < segments:
            cv = f"s{s}_cv"
            ops.append(_op(cv, "convert", main, dtype=dtype))     # transposes move stored values
            carry = f"s{s}_t"
            ops.append(_op(carry, "transpose", cv, perm=(1, 0)))
            r, c = c, r
        else:
            outputs.append((main, dtype))
    return GraphSpec(name=f"pattern_multi{seed}_{dtype}_{rows}x{cols}" + ("_ext" if external_links else ""), inputs=inputs, ops=ops,
                     outputs=outputs, external=external)


def independent_tiny_patterns_graph() -> GraphSpec:
    """One graph that holds eight small patterns with no edge between them and different row spaces (two row
    softmaxes, two residual LayerNorms, two RMSNorms, two softmax backwards): the explorer can only join them
    by packing their launches."""
    members = [softmax_graph(64, 128, "f32"), softmax_graph(96, 256, "f32"),
               add_bias_layernorm_graph(128, 768, in_dtype="bf16", out_dtype="bf16"),
               add_bias_layernorm_graph(48, 1024, in_dtype="bf16", out_dtype="bf16"),
               rmsnorm_graph(64, 2048, dtype="bf16"), rmsnorm_graph(40, 512, dtype="bf16"),
               softmax_backward_graph(384, 64, "f16"), softmax_backward_graph(100, 320, "f16")]
    inputs: List[TensorSpec] = []
    ops: List[OpSpec] = []
    outputs: List[Tuple[str, str]] = []
    for k, m in enumerate(members):
        ren = lambda n, k=k: f"s{k}_{n}"
        inputs += [TensorSpec(ren(t.name), t.dtype, t.dims) for t in m.inputs]
        ops += [OpSpec(ren(o.out), o.opcode, tuple(ren(i) for i in o.inputs), dict(o.attr)) for o in m.ops]
        outputs += [(ren(n), dt) for n, dt in m.outputs]
    return GraphSpec(name="pattern_independent_tiny", inputs=inputs, ops=ops, outputs=outputs)


def pack_members_p1() -> List[GraphSpec]:
    """P1: 32 independent tiny subgraphs (each a few microseconds or less on its own, so launch-bound when run
    one kernel each): the many-small-kernels regime that kernel packing addresses."""
    members: List[GraphSpec] = []
    members += [softmax_graph(64, 128, "f32") for _ in range(8)]                # the C1 shape
    members += [add_bias_layernorm_graph(128, 768) for _ in range(8)]
    members += [softmax_backward_graph(384, 128, "f16") for _ in range(8)]
    members += [rmsnorm_graph(64, 1024, dtype="bf16") for _ in range(4)]
    members += [bias_gelu_graph(64, 3072, "bf16") for _ in range(4)]
    return members


PACK_CONFIGS = {"P1": pack_members_p1}

# Multi-pattern graphs for the fusion explorer.
EXPLORE_CONFIGS = {"T1": lambda: transformer_block_graph(32, 128, 12, 64, 3072, "bf16"),
                   # the same block with the q/k/v projection biases added in front of the head split
                   "T2": lambda: transformer_block_graph(32, 128, 12, 64, 3072, "bf16", projection_bias=True),
                   # the backward pass through the block: row reductions, column sums and transposes side by side
                   "T3": lambda: transformer_block_backward_graph(32, 128, 12, 64, 3072, "bf16")}

# Row-local patterns outside the hand-written families, at transformer-block sizes (generated kernels; the interpreted row program beside them).
GENERIC_CONFIGS = {
    "G1": lambda: layernorm_stats_graph(8192, 768, with_variance=True),      # C2 plus mean / rstd / variance outputs
    "G2": lambda: silu_gate_graph(8192, 4096, "bf16"),
    "G3": lambda: scaled_softmax_colbias_graph(32 * 12 * 128, 128, "f32"),
    "G4": lambda: normalize_from_stats_graph(8192, 1024, "f16"),
    "G5": lambda: masked_scores_gate_graph(32, 12, 128, 128, "f16"),        # C3's shape: mask [B,1,1,T], per-head scale [H,1,1]
    # leading-axis transposes folded into a row kernel's load or store
    "G6": lambda: bias_head_split_graph(64, 512, 16, 64, "bf16"),            # projection bias + head split (store side)
    "G7": lambda: transpose_chain_stats_graph(64, 512, 12, 64),              # C5 plus the stored row sums (load side)
    "G8": lambda: head_merge_residual_graph(64, 512, 16, 64, "bf16"),        # head merge + gain + residual (load side)
    # column sums over all rows beside the row-local work: partial sums per workgroup + a fold launch
    "G9": lambda: gelu_backward_graph(16384, 3072, "bf16"),                  # C4's shape
    "G10": lambda: rmsnorm_backward_graph(8192, 4096, "bf16"),               # N5's shape
    # a row far beyond one workgroup's registers (probabilities over a vocabulary): chunks, a pass per row reduction
    "G11": lambda: softmax_graph(4096, 128256, "bf16"),
    "G12": lambda: log_softmax_graph(4096, 128256, "bf16"),                  # the same with a logarithm: what a cross-entropy reads
}

FULL_CONFIGS = {
    "C1": lambda: softmax_graph(64, 128, "f32"),
    "C2": lambda: add_bias_layernorm_graph(8192, 768),
    "C3": lambda: attention_scores_graph(32, 12, 128, 128),
    "C4": lambda: bias_gelu_dbias_graph(16384, 3072),
    "C5": lambda: transpose_chain_graph(64, 512, 12, 64),
}
