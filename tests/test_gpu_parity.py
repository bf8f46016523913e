"""GPU parity: every scheme and every enumerated launch shape of every pattern, plus the
per-op baseline, against the float64 oracle on the same seeded inputs.  Sizes span
several tiles and end in ragged tails.  All calls go through the C ABI."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2009_10924_amd import binding as B
from tests.gpu_util import TOL, all_candidates, check, note, run_spec
from workloads import (add_bias_layernorm_graph, attention_scores_graph, bias_gelu_dbias_graph, bias_gelu_graph,
                       layernorm_backward_graph, make_inputs, rmsnorm_graph, softmax_backward_graph, softmax_graph,
                       transpose_chain_graph, transpose_graph)
from workloads.graphs import GraphSpec, OpSpec, TensorSpec

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ C1 softmax
@pytest.mark.parametrize("rows,cols,dtype", [
    (64, 128, "f32"),        # the configuration itself
    (301, 128, "f32"),       # ragged row count across workgroups
    (37, 4, "f32"),          # one vector per row: a lane owns a row (thread composition)
    (19, 1000, "f32"),       # 250 vectors: partly filled lanes
    (7, 2048, "f32"),        # 512 vectors: fills 64 lanes x 8 vectors
    (5, 4096, "f32"),        # too long for a wavefront: workgroup per row
    (33, 37, "f32"),         # row not a multiple of 4: generic kernel
    (29, 264, "f16"), (29, 264, "bf16"),
])
def test_softmax(rows, cols, dtype):
    spec = softmax_graph(rows, cols, dtype)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    worst = all_candidates(spec, inp, ref, {}, repeat=2)
    note(f"softmax {rows}x{cols} {dtype}: worst rel err {worst}")


# ------------------------------------------------------------------ C3 attention scores
@pytest.mark.parametrize("B_,H,S,T,dtype", [(3, 2, 9, 128, "f16"), (2, 3, 5, 64, "f16"), (2, 2, 7, 40, "bf16"),
                                           (2, 2, 3, 128, "f32"), (2, 1, 4, 36, "f16")])
def test_attention_scores(B_, H, S, T, dtype):
    spec = attention_scores_graph(B_, H, S, T, dtype=dtype)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    all_candidates(spec, inp, ref, {})
    # masked keys come out as exact zeros
    got, _, _, _ = run_spec(spec, inp, "auto")
    assert ((got["y"] == 0) == (ref["y"] == 0)).all()


# ------------------------------------------------------------------ C2 add + bias + LayerNorm
@pytest.mark.parametrize("rows,cols,in_dt,out_dt", [
    (67, 768, "f32", "bf16"), (130, 768, "f32", "f32"), (9, 1024, "f32", "bf16"), (11, 100, "f32", "f32"),
    (5, 4, "f32", "f32"), (13, 2048, "f32", "f16"), (17, 768, "bf16", "bf16"), (17, 512, "f16", "f16"),
])
def test_add_bias_layernorm(rows, cols, in_dt, out_dt):
    spec = add_bias_layernorm_graph(rows, cols, in_dtype=in_dt, out_dtype=out_dt)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    floors = {"out": O.rms(ref["out"])}
    worst = all_candidates(spec, inp, ref, floors, repeat=2)
    note(f"layernorm {rows}x{cols} {in_dt}->{out_dt}: worst rel err (floor rms) {worst}")


def test_layernorm_variants_without_residual_or_affine():
    # plain LayerNorm (no residual, no bias), and normalisation without gamma / beta
    base = add_bias_layernorm_graph(21, 256, out_dtype="f32")
    inp = make_inputs(base, seed=0)
    plain_ops = [OpSpec("mu", "reduce_mean", ("x",), {"axis": 1}), OpSpec("c", "sub", ("x", "mu"))] + list(base.ops[4:10]) + \
                [OpSpec("o", "add", ("g", "beta"))]
    plain = GraphSpec("add_bias_layernorm_plain", [base.inputs[0], base.inputs[3], base.inputs[4]], plain_ops, [("o", "f32")])
    ref = O.evaluate(plain, inp)
    got, _, info, _ = run_spec(plain, inp, "auto")
    assert info["pattern"] == "layernorm"
    check(got["o"], ref["o"], "f32", O.rms(ref["o"]), "plain layernorm")
    noaff = GraphSpec("add_bias_layernorm_noaffine", base.inputs[:2], [base.ops[0]] +
                      [OpSpec("mu", "reduce_mean", ("h0",), {"axis": 1}), OpSpec("c", "sub", ("h0", "mu"))] + list(base.ops[4:9]),
                      [("n", "f32")])
    ref = O.evaluate(noaff, inp)
    got, _, info, _ = run_spec(noaff, inp, "auto")
    assert info["pattern"] == "layernorm"
    check(got["n"], ref["n"], "f32", O.rms(ref["n"]), "layernorm without affine")


# ------------------------------------------------------------------ C4 bias GELU + bias gradient
@pytest.mark.parametrize("rows,cols,dtype", [(300, 1032, "bf16"), (70, 512, "bf16"), (33, 264, "f16"), (129, 260, "f32"),
                                             (1, 8, "bf16")])
def test_bias_gelu_dbias(rows, cols, dtype):
    spec = bias_gelu_dbias_graph(rows, cols, dtype)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    floors = {"dbias": O.rms(ref["dbias"])}
    worst = all_candidates(spec, inp, ref, floors, repeat=3)
    note(f"bias_gelu_dbias {rows}x{cols} {dtype}: worst {worst}")


def test_bias_gelu_negative_tail():
    # z far below zero: the textbook 1+tanh(u) form cancels in float32, the kernel's form must not
    spec = bias_gelu_graph(4, 64, "f32")
    x = np.linspace(-5.0, -2.0, 256, dtype=np.float32).reshape(4, 64)
    inp = {"x": x, "bias": np.zeros(64, np.float32)}
    ref = O.evaluate(spec, inp)
    for scheme in ("unfused", "auto"):
        got, _, _, _ = run_spec(spec, inp, scheme)
        # float32 outputs carry the 1e-5 bar wherever the result is a normal float32
        normal = np.abs(ref["y"]) > 1e-30
        assert O.max_rel_err(got["y"][normal], ref["y"][normal]) <= 1e-5


def test_bias_gelu_only():
    for dtype in ("bf16", "f16", "f32"):
        spec = bias_gelu_graph(37, 520, dtype)
        inp = make_inputs(spec, seed=0)
        ref = O.evaluate(spec, inp)
        all_candidates(spec, inp, ref, {})


# ------------------------------------------------------------------ C5 transpose chain
@pytest.mark.parametrize("B_,S,H,D,dtype", [(2, 37, 12, 64, "f32"), (1, 5, 3, 128, "f32"), (3, 18, 5, 32, "f32"),
                                           (2, 9, 4, 256, "f32"), (2, 11, 12, 64, "bf16"), (1, 70, 2, 8, "f32")])
def test_transpose_chain(B_, S, H, D, dtype):
    spec = transpose_chain_graph(B_, S, H, D, dtype=dtype)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    worst = all_candidates(spec, inp, ref, {})
    note(f"transpose_chain {B_}x{S}x{H}x{D} {dtype}: worst {worst}")


# ------------------------------------------------------------------ backward patterns
# Their outputs are differences of nearly equal terms (dy - sum y dy; g - mean g - ...), so the
# rms floor applies as for the LayerNorm output.
@pytest.mark.parametrize("rows,cols,dtype", [(301, 128, "f32"), (64, 128, "f16"), (37, 4, "f32"), (19, 1000, "f32"),
                                             (7, 1024, "bf16"), (33, 37, "f32"), (5, 4096, "f32")])
def test_softmax_backward(rows, cols, dtype):
    spec = softmax_backward_graph(rows, cols, dtype)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    worst = all_candidates(spec, inp, ref, {"dx": O.rms(ref["dx"])}, repeat=2)
    note(f"softmax backward {rows}x{cols} {dtype}: {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(67, 4096, "bf16"), (130, 768, "f32"), (9, 1024, "f16"), (11, 100, "f32"),
                                             (5, 4, "f32"), (3, 8192, "bf16"), (33, 37, "f32")])
def test_rmsnorm(rows, cols, dtype):
    spec = rmsnorm_graph(rows, cols, dtype=dtype)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    worst = all_candidates(spec, inp, ref, {}, repeat=2)       # no cancellation: strict relative error
    note(f"rmsnorm {rows}x{cols} {dtype}: {worst}")


@pytest.mark.parametrize("rows,cols,dtype", [(67, 768, "f32"), (300, 256, "f32"), (9, 1024, "bf16"), (11, 100, "f32"),
                                             (5, 4, "f32"), (130, 520, "f16"), (1, 8, "f32"), (1030, 64, "f32")])
def test_layernorm_backward(rows, cols, dtype):
    spec = layernorm_backward_graph(rows, cols, dtype)
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    floors = {k: O.rms(ref[k]) for k in ("dx", "dgamma", "dbeta")}
    worst = all_candidates(spec, inp, ref, floors, repeat=2)
    note(f"layernorm backward {rows}x{cols} {dtype}: {worst}")


@pytest.mark.parametrize("rows,cols,in_dt,out_dt", [(100, 768, "f32", "bf16"), (37, 100, "f32", "f32"), (9, 1024, "bf16", "bf16"),
                                                   (5, 4096, "f32", "f32"), (300, 64, "f16", "f16"), (1, 8, "f32", "f32")])
def test_layernorm_with_saved_statistics(rows, cols, in_dt, out_dt):
    from workloads import layernorm_stats_graph
    spec = layernorm_stats_graph(rows, cols, in_dtype=in_dt, out_dtype=out_dt)
    assert B.Plan(B.Graph.from_spec(spec), "auto").info["pattern"] == "layernorm"
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    worst = all_candidates(spec, inp, ref, {"out": O.rms(ref["out"]), "mu": O.rms(ref["mu"])}, repeat=2)
    note(f"LayerNorm + mean/rstd outputs {rows}x{cols} {in_dt}->{out_dt}: {worst}")


# ------------------------------------------------------------------ transpose: bit-exact
@pytest.mark.parametrize("dims,perm,dtype", [
    ((4, 37, 12, 64), (0, 2, 1, 3), "f32"), ((3, 5, 7, 6), (0, 2, 1, 3), "i32"), ((2, 33, 5, 8), (2, 0, 1, 3), "bf16"),
    ((2, 9, 50, 70), (0, 1, 3, 2), "f32"), ((5, 40, 70), (2, 0, 1), "f16"), ((3, 4, 35, 33), (3, 1, 0, 2), "i32"),
    ((67, 129), (1, 0), "f32"), ((2, 3, 4, 5), (3, 2, 1, 0), "f32"), ((6, 10), (0, 1), "f32"),
    # both tile axes multiples of a 128-bit vector: the 64x64 vectorised LDS tile, with ragged tiles
    ((4, 40, 12, 64), (0, 2, 3, 1), "f32"), ((3, 24, 5, 16), (0, 2, 3, 1), "bf16"), ((2, 3, 72, 200), (0, 1, 3, 2), "f16"),
    ((132, 68), (1, 0), "i32"), ((2, 136, 3, 8), (3, 2, 0, 1), "f32"), ((64, 64), (1, 0), "bf16"),
])
def test_transpose_bit_exact(dims, perm, dtype):
    spec = transpose_graph(dims, perm, dtype)
    inp = make_inputs(spec)                     # element i carries the bit pattern of i
    want = np.ascontiguousarray(np.transpose(inp["x"], perm))
    for scheme in ("unfused", "auto"):
        note(f"  case {spec.name} scheme={scheme}")
        _, raw, info, _ = run_spec(spec, inp, scheme)
        assert raw["t"].shape == want.shape
        assert np.array_equal(raw["t"].view(np.uint8), want.view(np.uint8)), f"{spec.name} {info['kernel']}"
    # transpose o transpose = identity when the permutation is an involution
    if tuple(np.argsort(perm)) == tuple(perm):
        spec2 = transpose_graph(want.shape, perm, dtype)
        _, raw2, _, _ = run_spec(spec2, {"x": want}, "auto")
        assert np.array_equal(raw2["t"].view(np.uint8), inp["x"].view(np.uint8))


# ------------------------------------------------------------------ per-op plan on graphs no stitched kernel covers
def test_unfused_generic_graph():
    rng = np.random.default_rng(3)
    spec = GraphSpec("custom", [TensorSpec("a", "f32", (3, 5, 8)), TensorSpec("b", "f16", (5, 1)), TensorSpec("c", "bf16", (3, 1, 8))], [
        OpSpec("t0", "mul", ("a", "b")), OpSpec("t1", "max", ("t0", "c")), OpSpec("t2", "tanh", ("t1",)),
        OpSpec("t3", "reduce_max", ("t2",), {"axis": 1}), OpSpec("t4", "broadcast", ("t3",), {"dims": (3, 5, 8)}),
        OpSpec("t5", "div", ("t2", "t4")), OpSpec("t6", "reduce_mean", ("t5",), {"axis": 0}),
        OpSpec("t7", "convert", ("t5",), {"dtype": "f16"}), OpSpec("t8", "scale", ("t7",), {"value": 3.0}),
        OpSpec("t9", "transpose", ("t8",), {"perm": (2, 0, 1)}), OpSpec("t10", "add_scalar", ("t9",), {"value": -1.5}),
    ], [("t6", "f32"), ("t10", "f32"), ("t5", "bf16")])
    from workloads import quantise
    inp = {"a": quantise(rng.standard_normal((3, 5, 8)), "f32"), "b": quantise(rng.uniform(0.5, 2, (5, 1)), "f16"),
           "c": quantise(rng.standard_normal((3, 1, 8)), "bf16")}
    ref = O.evaluate(spec, inp)
    got, _, info, _ = run_spec(spec, inp, "auto")
    assert info["scheme"] == "unfused"
    check(got["t6"], ref["t6"], "f32", O.rms(ref["t6"]), "t6")
    check(got["t10"], ref["t10"], "f16", 0.0, "t10")       # passed through an explicit f16 rounding
    check(got["t5"], ref["t5"], "bf16", 0.0, "t5")


def test_execute_argument_errors():
    import torch
    spec = bias_gelu_dbias_graph(40, 64)
    inp = make_inputs(spec)
    g = B.Graph.from_spec(spec)
    plan = B.Plan(g, "global")
    dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
    dev_out = B.alloc_outputs(spec)
    with pytest.raises(B.FsError) as e:
        plan.execute(dev_in, dev_out, None)
    assert e.value.code == -7                                 # FS_ERR_WORKSPACE
    ws = plan.make_workspace()
    with pytest.raises(B.FsError) as e:
        plan.execute_ptrs([t.data_ptr() for t in dev_in], [dev_out[0].data_ptr() + 2, dev_out[1].data_ptr()],
                          ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
    assert e.value.code == -8                                 # FS_ERR_ALIGN
    plan.execute(dev_in, dev_out, ws)                         # still works afterwards
    torch.cuda.synchronize()


def test_degenerate_extents():
    """Rows of one or two elements, a single row, a single head: every plan the library offers for such a shape (a
    family's catch-all kernel, a generated kernel with single-element steps, or the per-op plan) against the oracle.
    A softmax over one element is 1, a LayerNorm over one element is beta, a column sum over one row is the row."""
    from tests.gpu_util import floors_for
    from workloads import layernorm_backward_graph, rmsnorm_graph, softmax_backward_graph
    cases = [softmax_graph(1, 1, "f32"), softmax_graph(7, 1, "f16"), softmax_graph(1, 2, "f32"), add_bias_layernorm_graph(3, 1),
             add_bias_layernorm_graph(1, 2), bias_gelu_dbias_graph(1, 8), bias_gelu_dbias_graph(5, 1), bias_gelu_dbias_graph(1, 1),
             transpose_chain_graph(2, 1, 3, 8), transpose_chain_graph(1, 1, 1, 4), transpose_chain_graph(3, 5, 1, 1),
             rmsnorm_graph(1, 1), softmax_backward_graph(1, 1, "f32"), layernorm_backward_graph(1, 4), layernorm_backward_graph(2, 1)]
    for spec in cases:
        inp = make_inputs(spec, seed=6)
        ref = O.evaluate(spec, inp)
        worst = all_candidates(spec, inp, ref, floors_for(spec, inp, ref), repeat=2)
        note(f"{spec.name}: worst {worst}")
    one = O.evaluate(softmax_graph(7, 1, "f16"), make_inputs(softmax_graph(7, 1, "f16"), seed=6))["y"]
    assert np.array_equal(one, np.ones_like(one))


def test_workspace_contents_on_entry_do_not_matter():
    """A workspace holds no counters and nothing that has to start at zero: the same plan run on a zeroed workspace and
    on one filled with 0xFF bytes (NaN as float32) gives bit-identical outputs -- column partial sums (the gelu and
    LayerNorm-backward families, a generated kernel with column sums), a per-op plan's intermediates, an explored
    program with a joint fold."""
    import torch
    from workloads import gelu_backward_graph, transformer_block_backward_graph

    def outputs_with(plan_like, spec, dev_in, fill):
        dev_out = B.alloc_outputs(spec)
        for t in dev_out:
            t.view(torch.uint8).fill_(0xA5)
        ws = plan_like.make_workspace()
        if ws is not None:
            ws.fill_(fill)
        if isinstance(plan_like, B.Program):
            stream = torch.cuda.current_stream().cuda_stream
            plan_like.bind([t.data_ptr() for t in dev_in], [t.data_ptr() for t in dev_out], ws.data_ptr(), ws.numel(), stream)()
        else:
            plan_like.execute(dev_in, dev_out, ws)
        torch.cuda.synchronize()
        return [t.view(torch.uint8).cpu().numpy().copy() for t in dev_out]

    cases = [(bias_gelu_dbias_graph(300, 1024), "auto"), (layernorm_backward_graph(130, 768, "f32"), "auto"),
             (gelu_backward_graph(200, 512, "bf16"), "auto"), (add_bias_layernorm_graph(70, 768), "unfused")]
    for spec, scheme in cases:
        plan = B.Plan(B.Graph.from_spec(spec), scheme)
        assert plan.info["workspace_bytes"] > 0, spec.name
        inp = make_inputs(spec, seed=2)
        dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
        a, b = outputs_with(plan, spec, dev_in, 0), outputs_with(plan, spec, dev_in, 0xFF)
        assert all(np.array_equal(x, y) for x, y in zip(a, b)), (spec.name, plan.info["kernel"])
    spec = transformer_block_backward_graph(2, 64, 4, 64, 512, "bf16")
    prog = B.Program(B.Graph.from_spec(spec))
    assert prog.info["workspace_bytes"] > 0
    inp = make_inputs(spec, seed=2)
    dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
    a, b = outputs_with(prog, spec, dev_in, 0), outputs_with(prog, spec, dev_in, 0xFF)
    assert all(np.array_equal(x, y) for x, y in zip(a, b)), "explored program"


def test_two_plans_on_two_streams_at_once():
    """fs_execute is re-entrant for different plans: two plans with workspaces of their own, issued alternately on two
    streams (default priority) so that their kernels overlap on the device, give what each gives alone."""
    import torch
    specs = [bias_gelu_dbias_graph(2048, 3072), layernorm_backward_graph(2048, 768, "f32")]
    plans = [B.Plan(B.Graph.from_spec(s), "auto") for s in specs]
    ins = [[B.to_device(make_inputs(s, seed=4)[t.name], t.dtype) for t in s.inputs] for s in specs]
    wss = [p.make_workspace() for p in plans]

    def run(on_streams):
        outs = [B.alloc_outputs(s) for s in specs]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()] if on_streams else [torch.cuda.current_stream()] * 2
        torch.cuda.synchronize()
        for _ in range(25):
            for k in (0, 1):
                plans[k].execute(ins[k], outs[k], wss[k], stream=streams[k].cuda_stream)
        torch.cuda.synchronize()
        return [[t.view(torch.uint8).cpu().numpy().copy() for t in o] for o in outs]

    alone, together = run(False), run(True)
    for a, b, s in zip(alone, together, specs):
        assert all(np.array_equal(x, y) for x, y in zip(a, b)), s.name

