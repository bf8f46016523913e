"""GPU parity of the generic stitched path (patterns no hand-written kernel family covers) in both its
forms, the interpreted row program and the kernel generated for the pattern: every enumerated launch
shape of either, plus the per-op plan, against the float64 oracle; named patterns and seeded random
patterns."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2009_10924_amd import binding as B
from tests.gpu_util import all_candidates, floors_for, note
from workloads import (bias_head_split_graph, gelu_backward_graph, head_merge_residual_graph, layernorm_backward_bias_graph,
                       layernorm_stats_graph, make_inputs,
                       rmsnorm_backward_graph,
                       normalize_from_stats_graph, outer_scale_graph, random_row_pattern, scaled_softmax_colbias_graph,
                       silu_gate_graph, transpose_chain_stats_graph, transposed_softmax_graph)

pytestmark = pytest.mark.gpu


def _run(spec, seed=0, repeat=2):
    info = B.Plan(B.Graph.from_spec(spec), "auto").info
    assert info["pattern"] in ("row_program", "row_generated"), (spec.name, info["pattern"])
    inp = make_inputs(spec, seed=seed)
    ref = O.evaluate(spec, inp)
    # the rms floor only where the descriptor says the output is a cancelling sum or difference; strict elsewhere
    worst = all_candidates(spec, inp, ref, floors_for(spec, inp, ref), repeat=repeat)
    return worst, info


@pytest.mark.parametrize("rows,cols,in_dt,out_dt", [(100, 768, "f32", "bf16"), (37, 100, "f32", "f32"), (9, 1024, "bf16", "bf16"),
                                                   (5, 4096, "f32", "f16"), (300, 64, "f16", "f32"), (3, 2048, "f16", "f16")])
def test_layernorm_with_saved_statistics(rows, cols, in_dt, out_dt):
    worst, info = _run(layernorm_stats_graph(rows, cols, in_dtype=in_dt, out_dtype=out_dt, with_variance=True))
    note(f"LayerNorm + statistics {rows}x{cols} {in_dt}->{out_dt}: {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(33, 1024, "bf16"), (257, 40, "f32"), (2, 8192, "f16"), (64, 128, "f32")])
def test_silu_gate(rows, cols, dtype):
    worst, _ = _run(silu_gate_graph(rows, cols, dtype))
    note(f"gated SiLU {rows}x{cols} {dtype}: {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(50, 128, "f32"), (7, 1000, "f32"), (19, 264, "f16"), (4, 4096, "bf16")])
def test_softmax_with_column_operands(rows, cols, dtype):
    worst, _ = _run(scaled_softmax_colbias_graph(rows, cols, dtype))
    note(f"softmax with column bias and gain {rows}x{cols} {dtype}: {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(20, 256, "f16"), (130, 768, "f32"), (3, 4096, "bf16"), (1, 8, "f32")])
def test_normalize_from_saved_statistics_and_broadcast_outputs(rows, cols, dtype):
    worst, _ = _run(normalize_from_stats_graph(rows, cols, dtype))
    note(f"normalise from statistics {rows}x{cols} {dtype}: {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(50, 128, "f32"), (7, 1000, "bf16"), (19, 264, "f16"), (4, 4096, "f32"), (33, 127, "f32"),
                                             (3, 50257, "f32"), (2, 128256, "bf16")])
def test_log_sigmoid_relu_abs_sqrt_patterns(rows, cols, dtype):
    """Log-softmax, a sigmoid gate with a rectified branch, rows scaled by their L2 norm with their L1 norms stored:
    every launch shape of the generated kernel and of the interpreted program, and the per-op plan."""
    from workloads import l1_l2_scale_graph, log_softmax_graph, sigmoid_gate_graph
    if not B.codegen_available() and (cols > 8192 or cols % 4):
        pytest.skip("rows of this length exist as generated kernels only")
    for make in (log_softmax_graph, sigmoid_gate_graph, l1_l2_scale_graph):
        spec = make(rows, cols, dtype)
        worst, info = _run(spec)
        note(f"{spec.name}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("rows,cols", [(7, 64), (300, 1024), (2, 4096)])
def test_outer_product_without_full_input(rows, cols):
    worst, _ = _run(outer_scale_graph(rows, cols))
    note(f"outer scale {rows}x{cols}: {worst}")


@pytest.mark.parametrize("dims,dtype", [((3, 2, 9, 128), "f16"), ((2, 3, 5, 64), "f32"), ((2, 2, 7, 40), "bf16"), ((4, 1, 3, 1024), "f16"),
                                        ((32, 12, 128, 128), "f16")])
def test_operands_stretched_along_leading_axes(dims, dtype):
    from workloads import masked_scores_gate_graph
    worst, info = _run(masked_scores_gate_graph(*dims, dtype=dtype))
    note(f"masked, per-head scaled, soft-capped softmax {dims} {dtype}: {info['kernel']}, worst {worst}")


@pytest.mark.parametrize("dims,dtype", [((2, 40, 3, 64), "bf16"), ((3, 7, 5, 16), "f32"), ((2, 130, 4, 128), "f16"), ((1, 33, 2, 1024), "f32")])
def test_transposes_folded_into_loads_and_stores(dims, dtype):
    """[B,S,H,D] <-> [B,H,S,D] around element-wise work and row reductions: the transposes cost no instruction,
    only the row addressing of a load or of the store changes."""
    for make in (bias_head_split_graph, head_merge_residual_graph, transposed_softmax_graph):
        worst, info = _run(make(*dims, dtype=dtype))
        note(f"{make.__name__} {dims} {dtype}: {info['n_candidates']} shapes, worst {worst}")
    worst, _ = _run(transpose_chain_stats_graph(*dims, dtype=dtype))
    note(f"transpose chain + stored row sums {dims} {dtype}: worst {worst}")


def test_folded_transposes_move_values_exactly():
    """x + 0 through a store-side transpose, and a load-side transpose times 1: what arrives is bit-identical to
    numpy's transpose of the input (float32, bfloat16 and float16 values survive the trip through float32 lanes)."""
    import torch
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    from tests.gpu_util import run_spec
    for dtype in ("f32", "bf16", "f16"):
        for perm in ((0, 2, 1, 3), (2, 0, 1, 3)):
            dims = (3, 5, 4, 64)
            store = GraphSpec(f"pattern_exact_store_{dtype}", [TensorSpec("x", dtype, dims)],
                              [OpSpec("z", "add_scalar", ("x",), {"value": 0.0}), OpSpec("zc", "convert", ("z",), {"dtype": dtype}),
                               OpSpec("out", "transpose", ("zc",), {"perm": perm})],
                              [("out", dtype)])
            load = GraphSpec(f"pattern_exact_load_{dtype}", [TensorSpec("x", dtype, dims)],
                             [OpSpec("t", "transpose", ("x",), {"perm": perm}), OpSpec("out", "scale", ("t",), {"value": 1.0})],
                             [("out", dtype)])
            for spec in (store, load):
                inp = make_inputs(spec, seed=3)
                want = np.transpose(inp["x"], perm)
                n = B.Plan(B.Graph.from_spec(spec), "auto").info["n_candidates"]
                for i in range(n):
                    _, raw, info, _ = run_spec(spec, inp, "auto", candidate=i)
                    assert np.array_equal(raw["out"].view(np.uint8), np.ascontiguousarray(want).view(np.uint8)), (spec.name, perm, info["kernel"])


def test_several_leading_axis_moves_as_one_kernel():
    """Three tensors each moved [B,S,H,D] -> [B,H,S,D] and stored (the head split of q, k and v), one of them also
    computed on: one launch, every moved value bit-identical to numpy's transpose."""
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    from tests.gpu_util import run_spec
    perm = (0, 2, 1, 3)
    for dtype, dims in (("bf16", (2, 37, 3, 64)), ("f32", (3, 5, 4, 36)), ("f16", (1, 130, 2, 30))):
        spec = GraphSpec(f"pattern_three_moves_{dtype}", [TensorSpec(n, dtype, dims) for n in "qkv"],
                         [OpSpec("tq", "transpose", ("q",), {"perm": perm}), OpSpec("tk", "transpose", ("k",), {"perm": perm}),
                          OpSpec("tv", "transpose", ("v",), {"perm": perm}), OpSpec("e", "tanh", ("tv",))],
                         [("tq", dtype), ("tk", dtype), ("tv", dtype), ("e", dtype)])
        inp = make_inputs(spec, seed=5)
        ref = O.evaluate(spec, inp)
        plan = B.Plan(B.Graph.from_spec(spec), "auto")
        assert plan.info["n_kernels"] == 1 and plan.info["pattern"] in ("row_program", "row_generated")
        for i in range(plan.info["n_candidates"]):
            got, raw, info, _ = run_spec(spec, inp, "auto", candidate=i)
            for name, src in (("tq", "q"), ("tk", "k"), ("tv", "v")):
                want = np.ascontiguousarray(np.transpose(inp[src], perm))
                assert np.array_equal(raw[name].view(np.uint8), want.view(np.uint8)), (spec.name, name, info["kernel"])
            assert O.max_rel_err(got["e"], ref["e"], O.rms(ref["e"])) <= (1e-5 if dtype == "f32" else 1e-2)


@pytest.mark.parametrize("rows,cols,dtype", [(10, 50, "f32"), (9, 1001, "bf16"), (13, 36, "f16"), (70, 127, "f16"), (3, 3003, "f32"),
                                             (300, 6, "bf16")])
def test_row_lengths_that_allow_no_128_bit_access(rows, cols, dtype):
    """Rows that are no multiple of 8 (16-bit) or 4 elements: the generated kernels step by 4 elements with 64-bit
    accesses for the 16-bit operands, or by single elements; before, such patterns ran per op."""
    if not B.codegen_available():
        pytest.skip("these step widths exist as generated kernels only")
    for make in (lambda: layernorm_stats_graph(rows, cols, in_dtype=dtype, out_dtype=dtype, with_variance=True),
                 lambda: silu_gate_graph(rows, cols, dtype), lambda: scaled_softmax_colbias_graph(rows, cols, dtype),
                 lambda: random_row_pattern(rows + cols, rows, cols, dtype, n_ops=10)):
        spec = make()
        worst, info = _run(spec)
        assert info["pattern"] == "row_generated"
        note(f"{spec.name}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(37, 96, "f32"), (1000, 128, "bf16"), (4100, 64, "f16"), (300, 768, "f32"), (2500, 1024, "bf16"),
                                             (70, 4096, "f16"), (5000, 8, "f32")])
def test_column_sums_beside_row_work(rows, cols, dtype):
    """A column sum over all rows next to row-local outputs (backward of bias + GELU, backward of RMSNorm): partial
    sums per workgroup in the workspace, folded by a second launch; every launch shape and every number of rows per
    lane group, ragged row counts included, and bit-identical results from run to run."""
    if not B.codegen_available():
        pytest.skip("column sums inside a row pattern exist as generated kernels only")
    for make in (gelu_backward_graph, rmsnorm_backward_graph, layernorm_backward_bias_graph):
        spec = make(rows, cols, dtype)
        # (the bias gradient of the LayerNorm pattern sums dx after its rounding to the storage dtype: it is compared
        # with the exact sum of the dx this run stored, at the float32 bar)
        worst, info = _run(spec, repeat=3)
        assert info["pattern"] == "row_generated" and info["n_kernels"] == 2 and info["scheme"] == "global"
        note(f"{spec.name}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(8, 16384, "bf16"), (5, 32768, "f16"), (3, 20000, "f32"), (4, 24576, "bf16")])
def test_long_rows_on_workgroups_of_512_and_1024_threads(rows, cols, dtype):
    """Rows beyond 256 threads x 8 vectors: generated kernels put 512 or 1024 threads on a row (reductions through LDS
    over 8 or 16 wavefronts)."""
    if not B.codegen_available():
        pytest.skip("workgroups wider than 256 threads exist as generated kernels only")
    from workloads import softmax_graph
    for spec in (layernorm_stats_graph(rows, cols, in_dtype=dtype, out_dtype=dtype, with_variance=True), silu_gate_graph(rows, cols, dtype),
                 softmax_graph(rows, cols, dtype)):
        g = B.Graph.from_spec(spec)
        info = B.Plan(g, "auto").info
        if spec.name.startswith("softmax") and info["pattern"] == "softmax":
            continue                                    # the softmax family's own block kernel still holds this row
        assert info["pattern"] == "row_generated" and info["block"][0] in (512, 1024), (spec.name, info)
        inp = make_inputs(spec, seed=1)
        ref = O.evaluate(spec, inp)
        worst = all_candidates(spec, inp, ref, floors_for(spec, inp, ref), repeat=2)
        note(f"{spec.name}: {info['kernel']} on {info['block'][0]} threads, worst {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(4, 131072, "bf16"), (3, 50257, "f32"), (5, 70000, "f16"), (2, 128256, "bf16"), (3, 40000, "f32")])
def test_rows_beyond_a_workgroups_registers_are_worked_through_in_chunks(rows, cols, dtype):
    """Rows longer than 1024 threads x 8 steps (a softmax over a vocabulary): the generated kernel walks the row in
    chunks, one pass per row reduction and one for the stores; whole chunks and a ragged last one, 8-, 4- and
    1-element steps, column operands, two outputs."""
    if not B.codegen_available():
        pytest.skip("rows of this length exist as generated kernels only")
    from workloads import softmax_graph
    for spec in (softmax_graph(rows, cols, dtype), layernorm_stats_graph(rows, cols, in_dtype=dtype, out_dtype=dtype, with_variance=True),
                 scaled_softmax_colbias_graph(rows, cols, dtype), silu_gate_graph(rows, cols, dtype)):
        plan = B.Plan(B.Graph.from_spec(spec), "auto")
        info = plan.info
        assert info["pattern"] == "row_generated" and "chunks" in info["kernel"] and info["n_kernels"] == 1, (spec.name, info)
        inp = make_inputs(spec, seed=2)
        ref = O.evaluate(spec, inp)
        worst = all_candidates(spec, inp, ref, floors_for(spec, inp, ref), repeat=2)
        note(f"{spec.name}: {info['kernel']} on {info['block'][0]} threads, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("dtype,cols", [("f32", 50257), ("bf16", 70000)])
def test_running_maximum_pass_on_rows_built_to_break_it(dtype, cols):
    """Softmax and log-softmax over rows in chunks gather maximum and sum in one pass under a running maximum.  Rows
    made to stress exactly that: the maximum rising with every chunk (every chunk rescales the sum so far), falling
    (never), sitting in the last element, a first third and a last third masked with -10000 (their terms underflow
    against the later / earlier maximum), a range of +-30 (terms from e^-60 to 1), and a constant row."""
    if not B.codegen_available():
        pytest.skip("rows of this length exist as generated kernels only")
    from workloads import log_softmax_graph, softmax_graph
    from workloads.inputs import quantise
    # (float32 carries |x - max| * 6e-8 of relative error into an exponential: the ranges keep that under the 1e-5 bar)
    ramp = np.linspace(-25.0, 25.0, cols)
    noise = np.random.default_rng(11).normal(0.0, 1.0, cols)
    spike, head_masked, tail_masked = noise.copy(), noise.copy(), noise.copy()
    spike[-1] = 30.0
    head_masked[:cols // 3] = -10000.0
    tail_masked[-(cols // 3):] = -10000.0
    plain = [ramp, ramp[::-1], spike, np.random.default_rng(12).uniform(-30.0, 30.0, cols), np.full(cols, 3.25)]
    # log-softmax of a masked entry is about -10000, which would set the rms floor of the whole output: masked rows
    # go through softmax only (there they are exact zeros)
    for make, rows in ((softmax_graph, plain + [head_masked, tail_masked]), (log_softmax_graph, plain)):
        spec = make(len(rows), cols, dtype)
        assert "chunks" in B.Plan(B.Graph.from_spec(spec), "auto").info["kernel"]
        inp = {spec.inputs[0].name: quantise(np.stack(rows), dtype)}
        ref = O.evaluate(spec, inp)
        worst = all_candidates(spec, inp, ref, floors_for(spec, inp, ref), repeat=1, unfused=False)
        note(f"{spec.name} on adversarial rows: worst {worst}")


@pytest.mark.parametrize("seed", range(48))
def test_random_row_patterns(seed):
    dtype = ("f32", "f16", "bf16")[seed % 3]
    rows, cols = [(37, 128), (5, 1000), (130, 64), (3, 4096), (64, 520), (9, 2048)][seed % 6]
    if dtype != "f32" and cols % 8:
        cols = cols // 8 * 8
    spec = random_row_pattern(seed, rows, cols, dtype, n_ops=6 + seed % 14)
    worst, info = _run(spec, seed=seed, repeat=1)
    note(f"random pattern {seed} {rows}x{cols} {dtype}: {len(spec.ops)} ops -> {info['kernel']}, worst {worst}")


@pytest.mark.parametrize("dims,dtype", [((2, 3, 2, 70000), "bf16"), ((1, 2, 3, 40004), "f32")])
def test_rows_in_chunks_with_folded_transposes(dims, dtype):
    """The row addressing of a folded transpose (permuted row strides in a load, a permuted row in the store) is the
    same whether a row is handled at once or chunk by chunk."""
    if not B.codegen_available():
        pytest.skip("rows of this length exist as generated kernels only")
    for make in (bias_head_split_graph, head_merge_residual_graph, transposed_softmax_graph):
        spec = make(*dims, dtype=dtype)
        worst, info = _run(spec)
        assert info["pattern"] == "row_generated" and "chunks" in info["kernel"], (spec.name, info)
        note(f"{make.__name__} {dims} {dtype}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("dims,dtype", [((4, 50, 128), "bf16"), ((3, 7, 5, 64), "f32"), ((32, 128, 768), "bf16"), ((2, 2, 300, 256), "f16")])
def test_bias_gradient_as_a_chain_of_sums_over_the_leading_axes(dims, dtype):
    """[B,S,H] or [B,S,N,H] activations: the sums along axis 0, 1, ... are one column sum of the pattern's row space."""
    if not B.codegen_available():
        pytest.skip("column sums inside a row pattern exist as generated kernels only")
    from workloads import bias_gradient_chain_graph
    spec = bias_gradient_chain_graph(dims, dtype)
    worst, info = _run(spec, repeat=2)
    assert info["pattern"] == "row_generated" and info["n_kernels"] == 2 and info["scheme"] == "global"
    note(f"{spec.name}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("rows,cols,dtype,sum_dtype", [(1000, 128, "bf16", "bf16"), (300, 768, "f16", "f16"), (2500, 1024, "f32", "bf16"), (37, 96, "bf16", "f16")])
def test_column_sums_handed_out_in_16_bits(rows, cols, dtype, sum_dtype):
    """The fold launch rounds the float32 sum once, to the dtype the gradient is wanted in."""
    if not B.codegen_available():
        pytest.skip("column sums inside a row pattern exist as generated kernels only")
    for make in (gelu_backward_graph, layernorm_backward_bias_graph):
        spec = make(rows, cols, dtype, sum_dtype=sum_dtype)
        worst, info = _run(spec, repeat=2)
        assert info["pattern"] == "row_generated" and info["n_kernels"] == 2 and info["scheme"] == "global"
        note(f"{spec.name} sums as {sum_dtype}: {info['kernel']}, worst {worst}")
    # sums of different dtypes side by side: a fold each where neighbours differ, all in one launch
    from workloads.graphs import GraphSpec
    spec = layernorm_backward_bias_graph(rows, cols, dtype, sum_dtype=sum_dtype)
    mixed = GraphSpec(spec.name + "_mixed", spec.inputs, spec.ops, [(n, "f32" if n == "dgamma" else d) for n, d in spec.outputs])
    worst, info = _run(mixed, repeat=2)
    assert info["pattern"] == "row_generated" and info["n_kernels"] == 2


@pytest.mark.parametrize("seed", range(24))
def test_random_row_patterns_with_the_wider_vocabulary(seed):
    dtype = ("f32", "f16", "bf16")[seed % 3]
    rows, cols = [(37, 96), (130, 64), (64, 520), (9, 1001), (5, 20000), (300, 256)][seed % 6]
    spec = random_row_pattern(1500 + seed, rows, cols, dtype, n_ops=6 + seed % 10, more_ops=True, column_sums=(seed % 2) if cols % 4 == 0 and cols < 8192 else 0)
    if not B.codegen_available() and B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused":
        pytest.skip("this shape exists as a generated kernel only")
    worst, info = _run(spec, seed=seed)
    note(f"random pattern {seed} (wider vocabulary) {rows}x{cols} {dtype}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("seed", range(9))
def test_random_row_patterns_on_rows_worked_through_in_chunks(seed):
    """Seeded random patterns (wider vocabulary, several inputs and outputs, kept values) on rows beyond a workgroup's
    registers: every chunked shape, with and without chunks kept in registers, and the per-op plan."""
    if not B.codegen_available():
        pytest.skip("rows of this length exist as generated kernels only")
    dtype = ("bf16", "f32", "f16")[seed % 3]
    rows, cols = [(3, 70000), (2, 40004), (4, 66000)][seed % 3]
    spec = random_row_pattern(2500 + seed, rows, cols, dtype, n_ops=5 + seed % 7, more_ops=seed % 2 == 1)
    worst, info = _run(spec, seed=seed)
    assert "chunks" in info["kernel"], info
    note(f"random pattern {seed} in chunks {rows}x{cols} {dtype}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")


@pytest.mark.parametrize("seed", range(24))
def test_random_row_patterns_with_column_sums(seed):
    """Seeded random patterns of which one to three full-shaped values are also summed over all rows: every launch
    shape (rows per lane group, column tiles where no row reduction ties the columns together) and the per-op plan."""
    dtype = ("f32", "f16", "bf16")[seed % 3]
    rows, cols = [(37, 96), (130, 64), (64, 520), (300, 256), (1000, 128), (9, 1024)][seed % 6]
    spec = random_row_pattern(900 + seed, rows, cols, dtype, n_ops=6 + seed % 9, column_sums=1 + seed % 3)
    inp = make_inputs(spec, seed=seed)
    ref = O.evaluate(spec, inp)
    floors = {name: O.rms(ref[name]) for name, _ in spec.outputs}
    info = B.Plan(B.Graph.from_spec(spec), "auto").info
    if B.codegen_available():
        assert info["pattern"] == "row_generated" and info["scheme"] == "global", (spec.name, info)
    worst = all_candidates(spec, inp, ref, floors, repeat=2)
    note(f"random pattern {seed} with column sums {rows}x{cols} {dtype}: {info['kernel']}, {info['n_candidates']} shapes, worst {worst}")
