"""Packed launches: many independent patterns in one kernel (kernel packing across
patterns, paper Sections 4.1 and 5.3), each member compared with the float64 oracle
on the same seeded inputs."""
import numpy as np
import pytest

from oracle import oracle as O
from tests.gpu_util import check, floors_for, note, run_pack
from workloads import make_inputs
from workloads.graphs import (add_bias_layernorm_graph, bias_gelu_graph, rmsnorm_graph, softmax_backward_graph,
                              softmax_graph)

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["fixed", "generated"], autouse=True)
def pack_form(request):
    """Every test runs twice: with the fixed packed kernel (a table of members dispatched at run time) and with
    kernels generated for exactly the members."""
    from paper_2009_10924_amd import binding as B
    if request.param == "generated" and not B.codegen_available():
        pytest.skip("needs the run-time compiler")
    with B.codegen(request.param == "generated"):
        yield request.param

# outputs formed by cancelling sums or differences (named so by the descriptor) are judged against max(|ref|, rms(ref))


def _check_members(specs, seeds, repeat=2):
    inputs = [make_inputs(s, seed=seed) for s, seed in zip(specs, seeds)]
    got, info = run_pack(specs, inputs, repeat=repeat)
    worst = 0.0
    for i, (spec, inp, res) in enumerate(zip(specs, inputs, got)):
        ref = O.evaluate(spec, inp)
        for name, dt in spec.outputs:
            floor = floors_for(spec, inp, ref).get(name, 0.0)
            worst = max(worst, check(res[name], ref[name], dt, floor, f"member {i} {spec.name}/{name}") / (1e-5 if dt == "f32" else 1e-2))
    return worst, info


def test_pack_of_patterns_outside_the_fixed_forms(pack_form):
    """Masked softmax, several outputs, folded transposes, patterns of no family, odd row lengths: members of a
    generated pack only."""
    from paper_2009_10924_amd import binding as B
    from workloads import (attention_scores_graph, bias_head_split_graph, layernorm_stats_graph, masked_scores_gate_graph,
                           random_row_pattern, silu_gate_graph, transposed_softmax_graph)
    specs = [attention_scores_graph(2, 3, 16, 64), layernorm_stats_graph(30, 96, with_variance=True), bias_head_split_graph(2, 9, 3, 16, "bf16"),
             silu_gate_graph(9, 50, "f16"), random_row_pattern(5, 20, 64, "f32", n_ops=9), transposed_softmax_graph(2, 7, 3, 32, "f32"),
             masked_scores_gate_graph(2, 3, 5, 64, dtype="f16"), softmax_graph(5, 8192, "bf16"), random_row_pattern(11, 33, 40, "bf16", n_ops=12)]
    if pack_form == "fixed":
        with pytest.raises(B.FsError) as e:
            _check_members(specs, seeds=range(len(specs)))
        assert e.value.code == -5
        return
    inputs = [make_inputs(s, seed=seed) for seed, s in enumerate(specs)]
    got, info = run_pack(specs, inputs, repeat=2)
    assert info["generated"] == 1 and info["n_kernels"] == 1
    for i, (spec, inp, res) in enumerate(zip(specs, inputs, got)):
        ref = O.evaluate(spec, inp)
        for name, dt in spec.outputs:
            check(res[name], ref[name].reshape(res[name].shape), dt, floors_for(spec, inp, ref).get(name, 0.0), f"member {i} {spec.name}/{name}")
    note(f"generated pack of {len(specs)} members outside the fixed forms: {info['grid']} workgroups, vgprs {info['vgprs']}")


def test_pack_mixed_patterns_dtypes_and_shapes():
    # every packed form, every dtype pair, wave rows (1, 2, 4 vectors per lane), workgroup rows, ragged row counts
    specs = [
        softmax_graph(64, 128, "f32"), softmax_graph(37, 100, "f32"), softmax_graph(9, 1024, "f16"), softmax_graph(5, 8192, "bf16"),
        softmax_graph(3, 4, "f32"), softmax_graph(1, 2048, "f32"),
        add_bias_layernorm_graph(100, 768), add_bias_layernorm_graph(33, 256, in_dtype="bf16", out_dtype="bf16"),
        add_bias_layernorm_graph(7, 1024, in_dtype="f16", out_dtype="f16"), add_bias_layernorm_graph(19, 3072, in_dtype="f32", out_dtype="f32"),
        add_bias_layernorm_graph(2, 4096, in_dtype="f32", out_dtype="bf16"),
        rmsnorm_graph(50, 4096), rmsnorm_graph(11, 520, dtype="f16"), rmsnorm_graph(130, 64, dtype="f32"),
        softmax_backward_graph(77, 256, "f16"), softmax_backward_graph(300, 128, "f32"), softmax_backward_graph(3, 2048, "bf16"),
        bias_gelu_graph(33, 3072), bias_gelu_graph(17, 40, "f32"), bias_gelu_graph(4, 8192, "f16"),
    ]
    worst, info = _check_members(specs, seeds=range(len(specs)))
    assert info["n_kernels"] == 1 and info["n_members"] == len(specs)
    note(f"pack ({'generated' if info['generated'] else 'fixed'}) of {len(specs)} mixed members, {info['grid']} workgroups, vgprs {info['vgprs']}: worst error {worst:.3f} of the bar")


def test_pack_single_member_and_repeated_member():
    worst, info = _check_members([softmax_graph(64, 128, "f32")], seeds=[0])
    assert info["n_kernels"] == 1
    specs = [rmsnorm_graph(16, 1024)] * 3          # same plan shape three times, different data
    worst, _ = _check_members(specs, seeds=[1, 2, 3])
    note(f"single and repeated members: worst {worst:.3f} of the bar")


def test_pack_more_members_than_one_launch_holds():
    specs = [softmax_graph(8 + i, 64 + 4 * (i % 5), "f32") if i % 2 else softmax_backward_graph(5 + i, 128, "f32")
             for i in range(70)]
    worst, info = _check_members(specs, seeds=range(70), repeat=1)
    assert info["n_kernels"] == 3
    note(f"70 members in {info['n_kernels']} launches: worst {worst:.3f} of the bar")


def test_pack_layer_norm_variant_without_residual():
    import dataclasses
    full = add_bias_layernorm_graph(45, 512, in_dtype="f32", out_dtype="f32")
    # plain LayerNorm: drop the residual and bias adds, normalise x itself
    ops = [dataclasses.replace(op, inputs=tuple("x" if n == "h" else n for n in op.inputs)) for op in full.ops[2:]]
    plain = dataclasses.replace(full, inputs=[t for t in full.inputs if t.name in ("x", "gamma", "beta")], ops=ops)
    worst, _ = _check_members([plain, full], seeds=[4, 5])
    note(f"plain + full LayerNorm members: worst {worst:.3f} of the bar")
