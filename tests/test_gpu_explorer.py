"""GPU parity of explored programs: a multi-pattern graph is cut into fusion patterns by the explorer, every
pattern runs as its own stitched plan (or packed launch), tensors between patterns go through the workspace;
all graph outputs are compared with the float64 oracle evaluated on the whole graph."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2009_10924_amd import binding as B
from tests.gpu_util import MIN_NORMAL, TOL, floors_for, note, stored_converts
from workloads import EXPLORE_CONFIGS, make_inputs, random_multi_pattern, random_row_pattern, transformer_block_graph

pytestmark = pytest.mark.gpu


def run_program(spec, inputs_np, repeat=2, **opts):
    import torch
    g = B.Graph.from_spec(spec)
    prog = B.Program(g, **opts)
    dev_in = [B.to_device(inputs_np[t.name], t.dtype) for t in spec.inputs]
    dev_out = B.alloc_outputs(spec)
    for t in dev_out:
        t.fill_(float("nan"))
    ws = prog.make_workspace()
    stream = torch.cuda.current_stream().cuda_stream
    call = prog.bind([t.data_ptr() for t in dev_in], [t.data_ptr() for t in dev_out], ws.data_ptr(), ws.numel(), stream)
    results = []
    for _ in range(repeat):
        call()
        torch.cuda.synchronize()
        results.append({name: B.to_host(t, dt).copy() for (name, dt), t in zip(spec.outputs, dev_out)})
    for r in results[1:]:
        for name in r:
            assert np.array_equal(r[name].view(np.uint8), results[0][name].view(np.uint8)), f"{name}: not run-to-run identical"
    return {name: O.to_f64(results[0][name], dt) for name, dt in spec.outputs}, prog


def run_program_raw(spec, inputs_np, **opts):
    """run_program, also handing back the stored arrays (storage dtype) of the first run."""
    got, prog = run_program(spec, inputs_np, **opts)
    return got, prog


def compare(spec, seed=0, **opts):
    """Every graph output against the float64 oracle: strict relative error, the rms floor only for the outputs the
    descriptor shows to be cancelling sums or differences.  Outputs computed from a `convert` result that is itself a
    graph output (the gradients rounded on their way to a matrix product) are compared with the oracle evaluated on
    the values the program stored for that result, at their own bar."""
    inp = make_inputs(spec, seed=seed)
    got, prog = run_program(spec, inp, **opts)
    names = stored_converts(spec)
    ref = O.evaluate(spec, inp, stored={n: got[n] for n in names}) if names else O.evaluate(spec, inp)
    floors = floors_for(spec, inp, ref)
    worst = 0.0
    for name, dt in spec.outputs:
        assert np.isfinite(got[name]).all(), f"{spec.name}/{name}: non-finite values"
        err = O.max_rel_err(got[name], ref[name].reshape(got[name].shape), max(floors.get(name, 0.0), MIN_NORMAL[dt]))
        assert err <= TOL[dt], f"{spec.name}/{name}: max rel err {err:.3e} > {TOL[dt]:.0e}"
        worst = max(worst, err / TOL[dt])
    return worst, prog


@pytest.mark.parametrize("dims", [(2, 16, 2, 8, 64), (3, 40, 4, 32, 256), (32, 128, 12, 64, 3072)])
def test_transformer_block(dims):
    spec = transformer_block_graph(*dims, "bf16")
    worst, prog = compare(spec)
    info = prog.info
    note(f"transformer block {dims}: {info['n_ops']} ops -> {info['n_patterns']} patterns + {info['n_single_ops']} single ops, "
         f"{info['n_kernels']} launches, {info['n_packs']} packs, workspace {info['workspace_bytes']} B, worst {worst:.3f} of the bar")
    # transposes are bit-exact copies of stored values
    inp = make_inputs(spec, seed=0)
    got, _ = run_program(spec, inp, repeat=1)
    want = O.to_f64(inp["q_lin"], "bf16").transpose(0, 2, 1, 3)
    assert np.array_equal(got["qt"], want)


@pytest.mark.parametrize("dims", [(2, 16, 2, 8, 64), (3, 40, 4, 32, 256), (32, 128, 12, 64, 3072)])
def test_transformer_block_with_projection_biases(dims):
    """Bias add + rounding + head split are three ops per projection: the explorer makes row patterns of them whose
    transposes are folded into the stores (generated kernels where the run-time compiler is there)."""
    spec = transformer_block_graph(*dims, "bf16", projection_bias=True)
    worst, prog = compare(spec)
    info = prog.info
    plans = [p["info"]["pattern"] for p in prog.patterns()]
    note(f"transformer block with projection biases {dims}: {info['n_ops']} ops -> {info['n_kernels']} launches {plans}, worst {worst:.3f}")
    assert info["n_kernels"] <= 8 and "transpose" not in plans[:2]      # no lone head-split transposes are left
    inp = make_inputs(spec, seed=0)
    got, _ = run_program(spec, inp, repeat=1)
    # the stored sum is the float32 sum of two bf16 values rounded once: compare exactly with that definition
    import torch
    q = torch.from_numpy(O.to_f64(inp["q_lin"], "bf16")).float() + torch.from_numpy(O.to_f64(inp["bias_q"], "bf16")).float()
    want = q.to(torch.bfloat16).float().numpy().transpose(0, 2, 1, 3)
    assert np.array_equal(got["qt"], want.astype(np.float64))


@pytest.mark.parametrize("dims", [(2, 16, 2, 8, 64), (3, 40, 4, 32, 256), (32, 128, 12, 64, 3072)])
def test_transformer_block_backward(dims):
    """Backward pass through the block: LayerNorm and GELU backward with their column sums (partial sums + fold launches
    inside generated kernels where the run-time compiler is there, per-op column reductions otherwise), softmax
    backward, gradient transposes; every output against the float64 oracle."""
    from workloads import transformer_block_backward_graph
    spec = transformer_block_backward_graph(*dims, "bf16")
    # (the bias gradients sum gradients that were rounded to bf16 on the way out, and LayerNorm 1's column sums start
    # from one: they are compared with the oracle evaluated on the rounded gradients this run stored)
    worst, prog = compare(spec)
    info = prog.info
    plans = [p["info"]["pattern"] for p in prog.patterns()]
    note(f"transformer block backward {dims}: {info['n_ops']} ops -> {info['n_patterns']} patterns + {info['n_single_ops']} single ops, "
         f"{info['n_kernels']} launches {plans}, workspace {info['workspace_bytes']} B, worst {worst:.3f} of the bar")
    assert info["n_kernels"] < info["n_ops"] // 2
    if B.codegen_available():
        # the folds that finish the column sums run as one launch behind the last step; the sums are the same bits
        assert info["n_joint_folds"] >= 4
        inp = make_inputs(spec, seed=0)
        joint, _ = run_program(spec, inp, repeat=1)
        apart, p2 = run_program(spec, inp, repeat=1, no_joint_folds=True)
        assert p2.info["n_joint_folds"] == 0 and p2.info["n_kernels"] > info["n_kernels"]
        for name, _ in spec.outputs:
            assert np.array_equal(joint[name], apart[name]), name


def _three_bias_gradients(rows, cols, dtype="f32"):
    """Three independent GELU-backward patterns over different row counts (so that they stay three patterns); the
    second one's bias gradient is read again (scaled) by a later op."""
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    inputs, ops, outputs = [], [], []
    for k in range(3):
        r = rows + 8 * k
        inputs += [TensorSpec(f"x{k}", dtype, (r, cols)), TensorSpec(f"b{k}", dtype, (cols,)), TensorSpec(f"g{k}", dtype, (r, cols))]
        ops += [OpSpec(f"z{k}", "add", (f"x{k}", f"b{k}")), OpSpec(f"d{k}", "gelu_tanh_grad", (f"z{k}",)),
                OpSpec(f"dx{k}", "mul", (f"g{k}", f"d{k}")), OpSpec(f"db{k}", "reduce_sum", (f"dx{k}",), {"axis": 0})]
        outputs += [(f"dx{k}", dtype), (f"db{k}", "f32")]
    ops.append(OpSpec("half", "scale", ("db1",), {"value": 0.5}))
    outputs.append(("half", "f32"))
    return GraphSpec(f"pattern_three_bias_gradients_{dtype}_{rows}x{cols}", inputs, ops, outputs)


@pytest.mark.parametrize("rows,cols", [(300, 256), (2100, 768)])
def test_folds_of_column_sums_that_are_read_again_stay_in_place(rows, cols):
    if not B.codegen_available():
        pytest.skip("column sums inside a pattern need the run-time compiler")
    spec = _three_bias_gradients(rows, cols)
    worst, prog = compare(spec)
    # db0 and db2 are finished by the joint launch at the end; db1 has a reader and is folded before it runs
    assert prog.info["n_joint_folds"] == 2
    _, apart = compare(spec, no_joint_folds=True)
    assert apart.info["n_kernels"] == prog.info["n_kernels"] + 1
    note(f"three bias gradients {rows}x{cols}: {prog.info['n_kernels']} launches ({apart.info['n_kernels']} with every fold in place), worst {worst:.3f}")


@pytest.mark.parametrize("backward", [False, True])
def test_block_runs_stage_by_stage_between_its_matrix_products(backward):
    """The block's graph names the matrix products that were taken out; the program has one stage per stretch between
    them.  Stage by stage, with the caller's work in between (here: re-writing the inputs the next stage reads, as
    the matrix product would), the outputs are those of the all-at-once run bit for bit."""
    import torch
    from workloads import transformer_block_backward_graph
    spec = (transformer_block_backward_graph if backward else transformer_block_graph)(3, 40, 4, 32, 256, "bf16")
    inp = make_inputs(spec, seed=3)
    whole, prog = run_program(spec, inp, repeat=1)
    assert prog.info["n_stages"] == 6
    dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
    late = {dst for _, dst in spec.external}                      # inputs that a matrix product hands over later
    for t, d in zip(spec.inputs, dev_in):
        if t.name in late:
            d.fill_(float("nan"))                                  # not there yet
    dev_out = B.alloc_outputs(spec)
    for o in dev_out:
        o.fill_(float("nan"))                                      # an output counts as made once it holds numbers
    ws = prog.make_workspace()
    stream = torch.cuda.current_stream().cuda_stream
    ins, outs = [t.data_ptr() for t in dev_in], [t.data_ptr() for t in dev_out]
    produced = set()
    for stage in range(prog.info["n_stages"]):
        prog.bind_stage(stage, ins, outs, ws.data_ptr(), ws.numel(), stream)()
        torch.cuda.synchronize()
        # the "matrix products" whose operands are complete hand over their results
        for (name, dt), o in zip(spec.outputs, dev_out):
            if not torch.isnan(o.float()).any():
                produced.add(name)
        for t, d in zip(spec.inputs, dev_in):
            if t.name in late and all(src in produced for src, dst in spec.external if dst == t.name):
                d.copy_(B.to_device(inp[t.name], t.dtype))
    for (name, dt), o in zip(spec.outputs, dev_out):
        got = O.to_f64(B.to_host(o, dt), dt)
        assert np.array_equal(got, whole[name]), name
    with pytest.raises(B.FsError):
        prog.bind_stage(6, ins, outs, ws.data_ptr(), ws.numel(), stream)()


@pytest.mark.parametrize("seed", range(8))
def test_random_programs_with_outside_links_run_stage_by_stage(seed):
    """Random segments, every other link of the chain a computation outside the graph: the program against the
    oracle, and stage by stage (the linked inputs filled in only once their source is complete) bit for bit the same."""
    import torch
    rows, cols = [(64, 128), (130, 64), (40, 520)][seed % 3]
    spec = random_multi_pattern(seed, rows=rows, cols=cols, segments=2 + seed % 3, external_links=True, column_sums=seed % 2)
    worst, prog = compare(spec, seed=seed)
    assert prog.info["n_stages"] == 1 + len(spec.external)        # the links are in series
    inp = make_inputs(spec, seed=seed)
    whole, _ = run_program(spec, inp, repeat=1)
    dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
    late = {dst: src for src, dst in spec.external}
    for t, d in zip(spec.inputs, dev_in):
        if t.name in late:
            d.fill_(float("nan"))
    dev_out = B.alloc_outputs(spec)
    for o in dev_out:
        o.fill_(float("nan"))
    ws = prog.make_workspace()
    stream = torch.cuda.current_stream().cuda_stream
    ins, outs = [t.data_ptr() for t in dev_in], [t.data_ptr() for t in dev_out]
    out_of = {name: o for (name, _), o in zip(spec.outputs, dev_out)}
    for stage in range(prog.info["n_stages"]):
        prog.bind_stage(stage, ins, outs, ws.data_ptr(), ws.numel(), stream)()
        torch.cuda.synchronize()
        for t, d in zip(spec.inputs, dev_in):
            if t.name in late and not torch.isnan(out_of[late[t.name]].float()).any() and torch.isnan(d.float()).any():
                d.copy_(B.to_device(inp[t.name], t.dtype))
    for (name, dt), o in zip(spec.outputs, dev_out):
        assert np.array_equal(O.to_f64(B.to_host(o, dt), dt), whole[name]), name
    note(f"multi pattern {seed} with outside links: {prog.info['n_stages']} stages, {prog.info['n_kernels']} launches, worst {worst:.3f} of the bar")


def test_block_forward_with_its_matrix_products_run_between_the_stages():
    """One encoder block end to end: the six stages of the explored program with the five groups of matrix products
    really run between them (torch, bfloat16) from the outputs the graph says they read.  Reference: the same flow in
    float64 with every stored tensor rounded to bfloat16.  A dependence missing from the graph's declaration would let
    a stage read an input before its matrix product wrote it (the inputs start out as NaN)."""
    import torch
    B_, S, H, Dh, F = 3, 40, 4, 32, 256
    hidden, rows = H * Dh, B_ * S
    spec = transformer_block_graph(B_, S, H, Dh, F, "bf16")
    prog = B.Program(B.Graph.from_spec(spec))
    assert prog.info["n_stages"] == 6
    rng = np.random.default_rng(7)

    def bf(a):                                   # float64 values on the bfloat16 grid
        return O.round_to(np.asarray(a, dtype=np.float64), "bf16")

    def store(v):                                # ... as storage (bit patterns)
        return (np.ascontiguousarray(v, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    x0 = bf(rng.standard_normal((rows, hidden)))
    W = {n: bf(rng.standard_normal(shape) / np.sqrt(shape[0])) for n, shape in
         (("q", (hidden, hidden)), ("k", (hidden, hidden)), ("v", (hidden, hidden)), ("o", (hidden, hidden)), ("1", (hidden, F)), ("2", (F, hidden)))}
    given = make_inputs(spec, seed=7)            # mask, biases, gains: the inputs no matrix product makes
    late = {dst for _, dst in spec.external} | {"q_lin", "k_lin", "v_lin", "x"}

    # what each matrix product computes, from float64 views of the tensors it reads (graph outputs and the block's input)
    products = {
        "q_lin": lambda t: (t["x0"] @ W["q"]).reshape(B_, S, H, Dh), "k_lin": lambda t: (t["x0"] @ W["k"]).reshape(B_, S, H, Dh),
        "v_lin": lambda t: (t["x0"] @ W["v"]).reshape(B_, S, H, Dh), "x": lambda t: t["x0"],
        "scores": lambda t: t["qt"] @ np.swapaxes(t["kt"], -1, -2), "ctx": lambda t: t["p_y"] @ t["vt"],
        "attn_out": lambda t: t["ctx_t"].reshape(rows, hidden) @ W["o"], "ffn1_out": lambda t: t["l1_out"] @ W["1"],
        "ffn2_out": lambda t: t["act"] @ W["2"],
    }
    needs = {"q_lin": [], "k_lin": [], "v_lin": [], "x": []}
    for src, dst in spec.external:
        needs.setdefault(dst, []).append(src)

    # reference: float64, one matrix product after the other in the order of the block, stored tensors rounded to
    # bfloat16.  Inputs that are not there yet are zeros: what does not depend on them is already right.
    dims = {t.name: t.dims for t in spec.inputs}
    ref_in = {t.name: (O.to_f64(given[t.name], t.dtype) if t.name not in late else np.zeros(t.dims)) for t in spec.inputs}
    seen = {"x0": x0}
    for name in ("q_lin", "k_lin", "v_lin", "x", "scores", "ctx", "attn_out", "ffn1_out", "ffn2_out"):
        assert all(src in seen for src in needs[name])
        ref_in[name] = bf(products[name](seen)).reshape(dims[name])
        out = O.evaluate(spec, {n: store(v) for n, v in ref_in.items()}, round_outputs=True)
        seen.update({n: out[n] for n, _ in spec.outputs})   # (those a later product reads are complete by then)
    ref = out

    # GPU: the program's stages with torch's matrix products between them
    dev_in = {t.name: (B.to_device(given[t.name], t.dtype) if t.name not in late else
                       torch.full(tuple(t.dims), float("nan"), dtype=torch.bfloat16, device="cuda")) for t in spec.inputs}
    dev_out = {name: o for (name, _), o in zip(spec.outputs, B.alloc_outputs(spec))}
    for o in dev_out.values():
        o.fill_(float("nan"))
    dW = {n: torch.from_numpy(w).to("cuda", torch.bfloat16) for n, w in W.items()}
    dx0 = torch.from_numpy(x0).to("cuda", torch.bfloat16)
    gpu_products = {
        "q_lin": lambda: (dx0 @ dW["q"]).view(B_, S, H, Dh), "k_lin": lambda: (dx0 @ dW["k"]).view(B_, S, H, Dh),
        "v_lin": lambda: (dx0 @ dW["v"]).view(B_, S, H, Dh), "x": lambda: dx0,
        "scores": lambda: dev_out["qt"] @ dev_out["kt"].transpose(-1, -2), "ctx": lambda: dev_out["p_y"] @ dev_out["vt"],
        "attn_out": lambda: dev_out["ctx_t"].reshape(rows, hidden) @ dW["o"], "ffn1_out": lambda: dev_out["l1_out"] @ dW["1"],
        "ffn2_out": lambda: dev_out["act"] @ dW["2"],
    }
    ws = prog.make_workspace()
    stream = torch.cuda.current_stream().cuda_stream
    ins = [dev_in[t.name].data_ptr() for t in spec.inputs]
    outs = [dev_out[name].data_ptr() for name, _ in spec.outputs]
    written = set()

    def run_products():
        for name in sorted(late - written):
            if all(not torch.isnan(dev_out[s].float()).any() for s in needs[name]):
                dev_in[name].copy_(gpu_products[name]())
                written.add(name)
    run_products()                               # the projections of the block's input
    for stage in range(prog.info["n_stages"]):
        prog.bind_stage(stage, ins, outs, ws.data_ptr(), ws.numel(), stream)()
        torch.cuda.synchronize()
        run_products()
    assert written == late
    for name, dt in spec.outputs:
        got = O.to_f64(B.to_host(dev_out[name], dt), dt)
        assert np.isfinite(got).all(), name
        # bfloat16 matrix products on the GPU accumulate in float32 and round once; the reference rounds float64
        # sums: a unit in the last place apart now and then, and LayerNorm passes that on
        err = O.max_rel_err(got, ref[name].reshape(got.shape), O.rms(ref[name]))
        assert err <= 5e-2, (name, err)
        note(f"    block forward with matrix products, {name}: max err {err:.2e} of the rms")


def test_a_stack_of_three_blocks_against_the_oracle():
    """Three blocks chained (a block's residual input is the previous block's output: an edge; its projections are
    declared matrix products): 111 ops, 18 launches in 18 stages, all at once against the oracle."""
    from workloads import transformer_stack_graph
    spec = transformer_stack_graph(3, 2, 16, 2, 8, 64, "bf16")
    worst, prog = compare(spec)
    assert prog.info["n_kernels"] == 18 and prog.info["n_stages"] == 18
    note(f"stack of 3 blocks: {prog.info['n_ops']} ops -> {prog.info['n_kernels']} launches, worst {worst:.3f} of the bar")


def test_transformer_block_without_packing_and_remote_fusion():
    spec = transformer_block_graph(2, 16, 2, 8, 64, "bf16")
    a, pa = compare(spec, no_packing=True)
    b, pb = compare(spec, no_remote_fusion=True, no_packing=True)
    note(f"small block: {pa.info['n_kernels']} launches without packing, {pb.info['n_kernels']} without remote fusion either")


@pytest.mark.parametrize("seed", range(24))
def test_random_multi_pattern_programs(seed):
    rows, cols = [(24, 32), (130, 64), (64, 520), (8, 1024)][seed % 4]
    spec = random_multi_pattern(seed, rows=rows, cols=cols, segments=2 + seed % 3)
    worst, prog = compare(spec, seed=seed)
    info = prog.info
    note(f"multi pattern {seed} {rows}x{cols}: {info['n_ops']} ops -> {info['n_kernels']} launches "
         f"({info['n_patterns']} patterns, {info['n_packs']} packs), workspace {info['workspace_bytes']} B, worst {worst:.3f} of the bar")


def _side_by_side(name, members):
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    inputs, ops, outputs = [], [], []
    for k, m in enumerate(members):
        ren = lambda n, k=k: f"s{k}_{n}"
        inputs += [TensorSpec(ren(t.name), t.dtype, t.dims) for t in m.inputs]
        ops += [OpSpec(ren(o.out), o.opcode, tuple(ren(i) for i in o.inputs), dict(o.attr)) for o in m.ops]
        outputs += [(ren(n), d) for n, d in m.outputs]
    return GraphSpec(name, inputs, ops, outputs)


def test_folds_of_hand_written_families_join_as_well():
    """Bias + GELU with its bias gradient (twice) and LayerNorm backward, side by side: three hand-written kernels
    with a fold launch each; the program issues the three folds as one launch."""
    from workloads import bias_gelu_dbias_graph, layernorm_backward_graph
    spec = _side_by_side("pattern_three_family_folds", [bias_gelu_dbias_graph(1000, 512), layernorm_backward_graph(600, 256, "f32"),
                                                         bias_gelu_dbias_graph(300, 1024)])
    inp = make_inputs(spec, seed=0)
    ref = O.evaluate(spec, inp)
    floors = floors_for(spec, inp, ref)
    got, prog = run_program(spec, inp)
    assert prog.info["n_joint_folds"] == 3 and prog.info["n_kernels"] == 4
    assert sorted(s["info"]["pattern"] for s in prog.patterns()) == ["bias_gelu_dbias", "bias_gelu_dbias", "layernorm_backward"]
    apart, p2 = run_program(spec, inp, no_joint_folds=True)
    assert p2.info["n_kernels"] == 6
    for name, dt in spec.outputs:
        assert np.array_equal(got[name], apart[name]), name
        err = O.max_rel_err(got[name], ref[name].reshape(got[name].shape), floors.get(name, 0.0))
        assert err <= TOL[dt], (name, err)


@pytest.mark.parametrize("seed", range(12))
def test_random_multi_pattern_programs_with_column_sums(seed):
    """Random segments that also sum one or two of their values over all rows: the folds of all segments run as one
    launch behind the last step (where two or more are free to move), and the result equals the one with every fold
    in place bit for bit."""
    rows, cols = [(64, 128), (130, 64), (40, 520)][seed % 3]
    spec = random_multi_pattern(seed, rows=rows, cols=cols, segments=2 + seed % 3, column_sums=1 + seed % 2)
    worst, prog = compare(spec, seed=seed)
    info = prog.info
    if B.codegen_available():
        inp = make_inputs(spec, seed=seed)
        joint, _ = run_program(spec, inp, repeat=1)
        apart, p2 = run_program(spec, inp, repeat=1, no_joint_folds=True)
        assert p2.info["n_joint_folds"] == 0
        for name, _ in spec.outputs:
            assert np.array_equal(joint[name], apart[name]), name
    note(f"multi pattern {seed} with column sums {rows}x{cols}: {info['n_ops']} ops -> {info['n_kernels']} launches "
         f"({info['n_joint_folds']} folds in the joint launch), worst {worst:.3f} of the bar")


@pytest.mark.parametrize("seed", range(8))
def test_single_pattern_graphs_through_the_explorer(seed):
    spec = random_row_pattern(500 + seed, 37, 128, ("f32", "f16", "bf16")[seed % 3], n_ops=6 + seed)
    worst, prog = compare(spec, seed=seed)
    note(f"row pattern {seed}: {prog.info['n_ops']} ops -> {prog.info['n_kernels']} launches, worst {worst:.3f}")


def test_independent_tiny_patterns_run_as_one_packed_launch():
    from workloads import independent_tiny_patterns_graph
    spec = independent_tiny_patterns_graph()
    worst, prog = compare(spec)
    assert prog.info["n_packs"] == 1 and prog.info["n_kernels"] == 1
    worst2, apart = compare(spec, no_packing=True)
    assert apart.info["n_kernels"] == 8
    note(f"eight independent tiny patterns: 1 packed launch (worst {worst:.3f} of the bar), 8 launches apart (worst {worst2:.3f})")


def test_program_execute_errors():
    import torch
    spec = random_multi_pattern(1)
    g = B.Graph.from_spec(spec)
    prog = B.Program(g)
    inp = make_inputs(spec)
    dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
    dev_out = B.alloc_outputs(spec)
    stream = torch.cuda.current_stream().cuda_stream
    if prog.info["workspace_bytes"] > 0:
        with pytest.raises(B.FsError) as e:
            prog.bind([t.data_ptr() for t in dev_in], [t.data_ptr() for t in dev_out], 0, 0, stream)()
        assert e.value.code == -7
    ws = prog.make_workspace()
    with pytest.raises(B.FsError) as e:
        prog.bind([t.data_ptr() for t in dev_in], [dev_out[0].data_ptr() + 4] + [t.data_ptr() for t in dev_out[1:]], ws.data_ptr(), ws.numel(), stream)()
    assert e.value.code == -8
    torch.cuda.synchronize()
