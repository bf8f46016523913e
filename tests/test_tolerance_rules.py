"""The rules the GPU parity tests judge by, checked on the CPU: which outputs get the rms floor (derived from the
descriptor), the smallest-normal floor of 16-bit outputs, and the reference for outputs computed from values the
graph itself rounded."""
import numpy as np

from oracle import oracle as O
from tests.gpu_util import MIN_NORMAL, cancelling_outputs, stored_converts
from workloads import (add_bias_layernorm_graph, attention_scores_graph, bias_gelu_dbias_graph, gelu_backward_graph,
                       layernorm_backward_bias_graph, layernorm_backward_graph, layernorm_stats_graph, log_softmax_graph, make_inputs,
                       rmsnorm_backward_graph, rmsnorm_graph, softmax_backward_graph, softmax_graph, transformer_block_backward_graph,
                       transformer_block_graph, transpose_chain_graph)
from workloads.graphs import GraphSpec, OpSpec, TensorSpec


def _names(spec):
    return cancelling_outputs(spec, make_inputs(spec, seed=0))


def test_rms_floor_goes_to_cancelling_sums_only():
    # the five configurations: the floor for the LayerNorm output and the bias gradient, strict for the rest
    assert _names(softmax_graph(8, 128, "f32")) == set()
    assert _names(add_bias_layernorm_graph(8, 768)) == {"out"}
    assert _names(attention_scores_graph(2, 2, 8, 128)) == set()
    assert _names(bias_gelu_dbias_graph(16, 64)) == {"dbias"}
    assert _names(transpose_chain_graph(2, 4, 3, 64)) == set()
    # backward patterns: differences and signed column sums
    assert _names(softmax_backward_graph(8, 128, "f16")) == {"dx"}
    assert _names(layernorm_backward_graph(8, 64, "f32")) == {"dx", "dgamma", "dbeta"}
    assert _names(gelu_backward_graph(16, 64, "bf16")) == {"dx", "dbias"}      # gelu' changes sign near z = -0.752
    assert _names(rmsnorm_backward_graph(8, 64, "bf16")) == {"dx", "dgamma"}
    # sums of squares and what is computed from them are strict; a row mean of signed values is not
    assert _names(rmsnorm_graph(8, 64, dtype="bf16")) == set()
    assert _names(layernorm_stats_graph(8, 64, with_variance=True)) == {"out", "mu"}
    # probabilities are strict, their logarithms (near zero for the row's largest entry) are not
    assert _names(softmax_graph(2, 1000, "bf16")) == set() and _names(log_softmax_graph(2, 1000, "bf16")) == {"y"}
    # the transformer block: only the two LayerNorm outputs; softmax probabilities, GELU and the moves are strict
    assert _names(transformer_block_graph(2, 16, 2, 8, 64, "bf16")) == {"l1_out", "l2_out"}
    back = _names(transformer_block_backward_graph(2, 16, 2, 8, 64, "bf16"))
    assert {"d_ctx", "d_q", "d_k", "d_v"}.isdisjoint(back) and {"l2_dxc", "dbias1", "l1_dgamma", "d_scores"} <= back


def test_sign_of_the_inputs_is_read_from_the_data():
    spec = GraphSpec("sum_of_inputs", [TensorSpec("x", "f32", (4, 8))],
                     [OpSpec("e", "scale", ("x",), {"value": 2.0}), OpSpec("s", "reduce_sum", ("e",), {"axis": 1})], [("s", "f32")])
    pos = {"x": np.abs(np.random.default_rng(0).standard_normal((4, 8))).astype(np.float32)}
    assert cancelling_outputs(spec, pos) == set()
    assert cancelling_outputs(spec, {"x": -pos["x"]}) == {"s"}


def test_smallest_normal_floor():
    # a float16 result of 3 subnormal steps stored as 2: relative error 1/3, absolute 6e-8; against the smallest normal
    # number (2^-14) that is 1e-3, inside the 1e-2 bar.  A normal float16 number gets no help from the floor.
    ref, got = np.array([3 * 2.0 ** -24]), np.array([2 * 2.0 ** -24])
    assert O.max_rel_err(got, ref, 0.0) > 0.3 and O.max_rel_err(got, ref, MIN_NORMAL["f16"]) < 1.1e-3
    ref, got = np.array([2.0 ** -13]), np.array([2.0 ** -13 * 1.02])
    assert O.max_rel_err(got, ref, MIN_NORMAL["f16"]) > 1e-2


def test_reference_given_stored_values_by_hand():
    # c = bf16(x); s = column sum of c.  With the values "some implementation" stored for c, s is their exact sum:
    # 1 + 2.015625 + 3 = 6.015625 (by hand), while the oracle's own c stays x un-rounded and its own s is 6.
    spec = GraphSpec("sum_after_rounding", [TensorSpec("x", "f32", (3, 1))],
                     [OpSpec("c", "convert", ("x",), {"dtype": "bf16"}), OpSpec("s", "reduce_sum", ("c",), {"axis": 0})],
                     [("c", "bf16"), ("s", "f32")])
    assert stored_converts(spec) == ["c"]
    inp = {"x": np.array([[1.0], [2.0], [3.0]], np.float32)}
    plain = O.evaluate(spec, inp)
    assert plain["s"].ravel().tolist() == [6.0]
    given = O.evaluate(spec, inp, stored={"c": np.array([[1.0], [2.015625], [3.0]])})
    assert given["s"].ravel().tolist() == [6.015625] and given["c"].ravel().tolist() == [1.0, 2.0, 3.0]
    # handing back the oracle's own rounding changes nothing
    spec2 = layernorm_backward_bias_graph(16, 64, "bf16")
    inp2 = make_inputs(spec2, seed=3)
    own = O.evaluate(spec2, inp2, round_outputs=True)
    again = O.evaluate(spec2, inp2, stored={"dxc": own["dxc"]})
    plain2 = O.evaluate(spec2, inp2)
    for name, _ in spec2.outputs:
        assert np.array_equal(again[name], plain2[name]), name
