"""Host compiler of the interpreted row program, checked on the CPU: the instruction listing the
library hands out (fs_plan_describe) is executed by a small numpy emulator written here and its
results are compared with the float64 oracle.  A wrong operand, a register reused too early or a
value dropped from the accumulator shows up as a numerical mismatch without any GPU."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2009_10924_amd import binding as B
from workloads import (l1_l2_scale_graph, log_softmax_graph, sigmoid_gate_graph, layernorm_stats_graph, make_inputs, normalize_from_stats_graph, outer_scale_graph,
                       random_row_pattern, scaled_softmax_colbias_graph, silu_gate_graph)

NP_DT = {0: "f32", 1: "f16", 2: "bf16"}


def _round_through(v, dt):
    if dt == "f32":
        return v.astype(np.float32)
    return O.to_f64(O.round_to(v.astype(np.float64), dt), dt).astype(np.float32)


def _gelu(z):
    z = z.astype(np.float64)
    return 0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))


def _gelu_grad(z):
    z = z.astype(np.float64)
    u = np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)
    t = np.tanh(u)
    return 0.5 * (1.0 + t) + 0.5 * z * (1.0 - t * t) * np.sqrt(2.0 / np.pi) * (1.0 + 3 * 0.044715 * z * z)


def emulate(listing, spec, inputs, anchor_dims):
    """Runs the listed program in float32 on whole arrays: full values [R, C], per-row values [R, 1].
    anchor_dims: extents of the pattern's row space (inputs stretched along leading axes are repeated to it)."""
    lines = [l.split() for l in listing.splitlines()]
    head = [l for l in lines if l and l[0] == "program"][0]
    kv = dict(x.split("=") for x in head[1:])
    rows, cols = int(kv["rows"]), int(kv["cols"])
    in_arrays = [O.to_f64(inputs[t.name], t.dtype).astype(np.float32) for t in spec.inputs]
    regs, sregs, outs, colvecs = {}, {}, {}, {}
    acc0 = None
    out_bind, rout_bind, out_rows = {}, {}, {}
    # the row's index along the (collapsed) leading axes, as the kernels derive it
    lead = [int(x) for x in kv["lead"].split(",")]
    r = np.arange(rows)
    c2, q1 = r % lead[2], r // lead[2]
    c1, c0 = q1 % lead[1], q1 // lead[1]

    def strided_rows(field):
        ms = [int(x) for x in field.split("=")[1].split(",")]
        return c0 * ms[0] + c1 * ms[1] + c2 * ms[2]

    for l in lines:
        if not l:
            continue
        if l[0] == "full":
            strides = [x for x in l if x.startswith("rowstrides=")]
            if strides:   # stretched along leading axes, or rows renumbered by a folded transpose: gather by row strides
                full = in_arrays[int(l[1][2:])].reshape(-1, cols)[strided_rows(strides[0])]
            else:
                full = in_arrays[int(l[1][2:])].reshape(rows, cols)
            if int(l[3]) != 255:
                regs[int(l[3])] = full
            if l[-1] == "acc":
                acc0 = full
        elif l[0] == "col":
            colvecs[int(l[3])] = np.broadcast_to(in_arrays[int(l[1][2:])].reshape(1, cols), (rows, cols))
        elif l[0] == "rscal":
            strides = [x for x in l if x.startswith("rowstrides=")]
            if strides:
                sregs[int(l[3])] = in_arrays[int(l[1][2:])].reshape(-1, 1)[strided_rows(strides[0])]
            else:
                sregs[int(l[3])] = in_arrays[int(l[1][2:])].reshape(rows, 1)
        elif l[0] == "output":
            out_bind[int(l[1])] = int(l[2][3:])
            strides = [x for x in l if x.startswith("rowstrides=")]
            if strides:   # stored through a folded transpose: scatter
                out_rows[int(l[1])] = strided_rows(strides[0])
        elif l[0] == "routput":
            rout_bind[int(l[1])] = int(l[2][3:])
    # column sums leave through the fold launch that follows: its pointer lines name the outputs
    fold = [i for i, l in enumerate(lines) if l[:2] == ["launch", "colfold"]]
    colsum_bind = {}
    handed = 0
    for k, start in enumerate(fold):          # each fold launch hands out one or two sums, in order
        mine = [l for l in lines[start + 1:(fold[k + 1] if k + 1 < len(fold) else len(lines))] if l and l[0] in ("ptr1", "ptr2")]
        for l in mine:
            colsum_bind[handed + int(l[0][3:]) - 1] = int(l[1][3:])
        handed += len(mine)
    acc = np.zeros((rows, cols), np.float32) if acc0 is None else acc0.copy()
    sacc = np.zeros((rows, 1), np.float32)
    f32 = np.float32
    n_instr = 0
    for l in lines:
        if not l or l[0] != "instr":
            continue
        n_instr += 1
        op = l[2]
        f = dict(x.split("=") for x in l[3:])
        imm = f32(float(f["imm"]))
        scalar, keep = f["flags"][0] == "s", f["flags"][1] == "k"
        aux = NP_DT[int(f["aux"])]
        dst = int(f["dst"])
        kind, idx = f["b"].split(":")
        if op == "store":
            if dst in out_rows:
                assert sorted(out_rows[dst]) == list(range(rows)), "the permuted store must write every row once"
                t = np.empty_like(acc)
                t[out_rows[dst]] = acc
                outs[out_bind[dst]] = t
            else:
                outs[out_bind[dst]] = acc.copy()
            continue
        if op == "store_scal":
            outs[rout_bind[dst]] = sacc.copy()
            continue
        if op == "colsum":
            outs[colsum_bind[dst]] = acc.astype(np.float64).sum(axis=0).astype(np.float32)
            continue
        if op in ("rsum", "rmax", "rsumsq"):
            src = acc * acc if op == "rsumsq" else acc
            sacc = (src.max(axis=1, keepdims=True) if op == "rmax" else src.sum(axis=1, keepdims=True, dtype=np.float32)).astype(f32)
            if keep:
                sregs[dst] = sacc
            continue
        b = {"acc": lambda: acc, "sacc": lambda: sacc, "reg": lambda: regs[int(idx)], "scal": lambda: sregs[int(idx)],
             "col": lambda: colvecs[int(idx)], "imm": lambda: np.full((1, 1), imm, np.float32)}[kind]()
        a = sacc if scalar else acc
        if scalar:
            assert kind in ("sacc", "scal", "imm"), "per-row instruction with a full-shaped operand"
        with np.errstate(all="ignore"):
            r = {"add": lambda: a + b, "sub": lambda: a - b, "rsub": lambda: b - a, "mul": lambda: a * b, "div": lambda: a / b,
                 "rdiv": lambda: b / a, "max": lambda: np.maximum(a, b), "square": lambda: a * a, "exp": lambda: np.exp(a),
                 "rsqrt": lambda: 1.0 / np.sqrt(a), "tanh": lambda: np.tanh(a), "gelu": lambda: _gelu(a),
                 "gelu_grad": lambda: _gelu_grad(a), "log": lambda: np.log(a), "sigmoid": lambda: 1.0 / (1.0 + np.exp(-a)),
                 "relu": lambda: np.maximum(a, 0.0), "abs": lambda: np.abs(a), "sqrt": lambda: np.sqrt(a), "load": lambda: b, "cvt": lambda: _round_through(a, aux)}[op]()
        r = np.asarray(r, dtype=np.float32)
        if scalar:
            sacc = np.broadcast_to(r, (rows, 1)).copy()
            if keep:
                sregs[dst] = sacc
        else:
            acc = np.broadcast_to(r, (rows, cols)).copy()
            if keep:
                regs[dst] = acc
    result = {}
    for slot, (name, dt) in enumerate(spec.outputs):
        result[name] = outs[slot].astype(np.float64)
    return result, n_instr


def _compare(spec, seed=1):
    plan = B.Plan(B.Graph.from_spec(spec), "auto")
    # the same instruction list drives the interpreter and the code generator; AUTO picks the generated kernel
    assert plan.info["pattern"] in ("row_program", "row_generated"), (spec.name, plan.info["pattern"])
    if plan.info["pattern"] == "row_generated":
        src = plan.source()
        assert "__global__ void __launch_bounds__(256) fs_gen_row_" in src and src.count("row.store") + src.count("colsum_flush") == len(spec.outputs)
    listing = plan.describe()
    inp = make_inputs(spec, seed=seed)
    ref = O.evaluate(spec, inp)
    anchor = max([ref[name].shape for name, _ in spec.outputs] + [tuple(t.dims) for t in spec.inputs], key=lambda d: int(np.prod(d)))
    got, n_instr = emulate(listing, spec, inp, anchor)
    for name, dt in spec.outputs:
        r = ref[name].reshape(got[name].shape)
        err = O.max_rel_err(got[name], r, O.rms(r))
        assert err < 2e-5, f"{spec.name}/{name}: emulated program is off by {err:.3e}\n{listing}"
    return n_instr, plan.info


@pytest.mark.parametrize("make", [
    lambda: layernorm_stats_graph(24, 96, in_dtype="f32", out_dtype="f32", with_variance=True),
    lambda: silu_gate_graph(9, 64, "f32"),
    lambda: scaled_softmax_colbias_graph(13, 40, "f32"),
    lambda: normalize_from_stats_graph(11, 48, "f32"),
    lambda: outer_scale_graph(7, 16),
    lambda: log_softmax_graph(11, 72, "f32"),
    lambda: sigmoid_gate_graph(9, 64, "f32"),
    lambda: l1_l2_scale_graph(13, 40, "f32"),
])
def test_named_patterns_compile_to_correct_programs(make):
    _compare(make())


def test_inputs_stretched_along_leading_axes():
    from workloads import masked_scores_gate_graph
    for dims in [(2, 3, 5, 16), (3, 1, 4, 32), (2, 2, 2, 8)]:
        n, info = _compare(masked_scores_gate_graph(*dims, dtype="f32"))
        assert info["pattern"] in ("row_program", "row_generated")


def _permuted(dims, perm):
    return tuple(dims[p] for p in perm)


@pytest.mark.parametrize("dims,perm", [
    ((2, 5, 3, 16), (0, 2, 1, 3)),    # head split / merge: an involution
    ((2, 5, 3, 16), (2, 0, 1, 3)),    # a rotation of the leading axes: perm and its inverse differ
    ((3, 2, 4, 8), (1, 2, 0, 3)),
    ((6, 4, 32), (1, 0, 2)),          # rank 3
    ((1, 7, 3, 8), (2, 1, 0, 3)),     # an extent of 1 among the permuted axes
])
def test_transposes_of_leading_axes_fold_into_loads_and_stores(dims, perm):
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    out_dims = _permuted(dims, perm)
    rank = len(dims)
    # load side: y = exp(tanh(transpose(x))) * g + res, all in the transposed space; the row sums are stored too
    load = GraphSpec(f"pattern_view_load_{'x'.join(map(str, dims))}_{''.join(map(str, perm))}",
                     [TensorSpec("x", "f32", dims), TensorSpec("g", "f32", (dims[-1],)), TensorSpec("res", "f32", out_dims)],
                     [OpSpec("t", "transpose", ("x",), {"perm": perm}), OpSpec("h", "tanh", ("t",)), OpSpec("e", "exp", ("h",)),
                      OpSpec("u", "mul", ("e", "g")), OpSpec("y", "add", ("u", "res")),
                      OpSpec("s", "reduce_sum", ("y",), {"axis": rank - 1})],
                     [("y", "f32"), ("s", "f32")])
    _, info = _compare(load)
    listing = B.Plan(B.Graph.from_spec(load), "auto").describe()
    assert "transpose" not in listing and "rowstrides=" in listing          # no instruction: the load's addressing does it
    # store side: z = x * r + bias, stored transposed; z's row maxima stored in the original order
    store = GraphSpec(f"pattern_view_store_{'x'.join(map(str, dims))}_{''.join(map(str, perm))}",
                      [TensorSpec("x", "f32", dims), TensorSpec("r", "f32", dims[:-1] + (1,)), TensorSpec("bias", "f32", dims[-2:])],
                      [OpSpec("a", "mul", ("x", "r")), OpSpec("z", "add", ("a", "bias")),
                       OpSpec("m", "reduce_max", ("z",), {"axis": rank - 1}), OpSpec("out", "transpose", ("z",), {"perm": perm})],
                      [("out", "f32"), ("m", "f32")])
    _compare(store)
    # both sides at once: transposed in, the inverse permutation out (only the arithmetic remains)
    inverse = tuple(perm.index(k) for k in range(rank))
    both = GraphSpec(f"pattern_view_both_{'x'.join(map(str, dims))}_{''.join(map(str, perm))}",
                     [TensorSpec("x", "f32", dims)],
                     [OpSpec("t", "transpose", ("x",), {"perm": perm}), OpSpec("q", "square", ("t",)),
                      OpSpec("out", "transpose", ("q",), {"perm": inverse})],
                     [("out", "f32")])
    _compare(both)


def test_transposed_views_that_are_outputs_compile_to_load_and_store():
    """A leading-axis transpose whose result is itself an output is a move: a load through the permuted row strides
    and a plain store, as many of them in one program as the operand limit allows."""
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    dims, perm = (2, 5, 3, 16), (0, 2, 1, 3)
    spec = GraphSpec("pattern_three_moves", [TensorSpec(n, "f32", dims) for n in "qkv"],
                     [OpSpec("tq", "transpose", ("q",), {"perm": perm}), OpSpec("tk", "transpose", ("k",), {"perm": perm}),
                      OpSpec("tv", "transpose", ("v",), {"perm": perm}), OpSpec("e", "exp", ("tv",))],
                     [("tq", "f32"), ("tk", "f32"), ("tv", "f32"), ("e", "f32")])
    n_instr, info = _compare(spec)
    assert info["n_kernels"] == 1 and n_instr <= 8
    listing = B.Plan(B.Graph.from_spec(spec), "auto").describe()
    assert listing.count("rowstrides=15,1,3") == 3 and listing.count(" store ") == 4


@pytest.mark.parametrize("dims", [(4, 9, 64), (2, 3, 5, 32), (37, 96)])
def test_sums_over_several_leading_axes_in_a_chain_are_one_column_sum(dims):
    from workloads import bias_gradient_chain_graph
    from workloads.graphs import GraphSpec
    if not B.codegen_available():
        pytest.skip("needs the run-time compiler")
    spec = bias_gradient_chain_graph(dims, "f32")
    n_instr, info = _compare(spec)
    assert info["n_kernels"] == 2 and n_instr == 5          # add, gelu', mul, store, colsum: the chain's links emit nothing
    if len(dims) > 2:
        # a chain that stops before the last leading axis leaves values that several rows share: no row program
        short = GraphSpec("pattern_short_chain", spec.inputs, spec.ops[:-1], [("dx", "f32"), (spec.ops[-2].out, "f32")])
        assert B.Plan(B.Graph.from_spec(short), "auto").info["scheme"] == "unfused"
        # and one whose link is read elsewhere as well
        extra = GraphSpec("pattern_read_link", spec.inputs, list(spec.ops) + [type(spec.ops[0])("h", "scale", ("s0",), {"value": 0.5})],
                          list(spec.outputs) + [("h", "f32")])
        assert B.Plan(B.Graph.from_spec(extra), "auto").info["scheme"] == "unfused"


def test_column_sums_of_different_dtypes_get_folds_of_their_own():
    """A fold rounds what it hands out to one dtype: two neighbouring sums of the same dtype share a fold, a sum whose
    neighbour has another dtype gets its own; the folds of one pattern go out as one launch."""
    from workloads import gelu_backward_graph, layernorm_backward_bias_graph
    from workloads.graphs import GraphSpec
    if not B.codegen_available():
        pytest.skip("needs the run-time compiler")
    plan = B.Plan(B.Graph.from_spec(gelu_backward_graph(64, 128, "bf16", sum_dtype="bf16")), "auto")
    assert plan.info["pattern"] == "row_generated" and plan.info["n_kernels"] == 2
    spec = layernorm_backward_bias_graph(64, 128, "f32", sum_dtype="bf16")          # dbias, dgamma, dbeta all bf16: 2 folds
    plan = B.Plan(B.Graph.from_spec(spec), "auto")
    assert plan.info["n_kernels"] == 2 and plan.describe().count("colfold") >= 2
    mixed = GraphSpec(spec.name + "_mixed", spec.inputs, spec.ops, [(n, "f32" if n == "dgamma" else d) for n, d in spec.outputs])
    n_instr, info = _compare(mixed)                                                     # bf16, f32, bf16: a fold each
    assert info["pattern"] == "row_generated" and info["n_kernels"] == 2


@pytest.mark.parametrize("rows,cols", [(37, 96), (50, 128), (9, 1024)])
def test_column_sums_compile_to_partial_sums_and_a_fold(rows, cols):
    from workloads import gelu_backward_graph, layernorm_backward_bias_graph, rmsnorm_backward_graph
    for make in (gelu_backward_graph, rmsnorm_backward_graph, layernorm_backward_bias_graph):
        spec = make(rows, cols, "f32")
        _, info = _compare(spec)
        if B.codegen_available():
            assert info["n_kernels"] == 2 and info["scheme"] == "global"    # the pattern's kernel, then its folds as one launch
            assert info["workspace_bytes"] % (cols * 4) == 0 and info["workspace_bytes"] > 0


def test_transposes_a_row_program_cannot_fold():
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    # the innermost axis moves: data crosses rows -> the pattern is not one row kernel
    spec = GraphSpec("pattern_inner", [TensorSpec("x", "f32", (4, 8, 16))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("t", "transpose", ("e",), {"perm": (0, 2, 1)})], [("t", "f32")])
    assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"
    # a transposed intermediate that is computed on afterwards: neither a load nor a store
    spec = GraphSpec("pattern_mid", [TensorSpec("x", "f32", (4, 8, 16))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("t", "transpose", ("e",), {"perm": (1, 0, 2)}), OpSpec("y", "tanh", ("t",))],
                     [("y", "f32")])
    assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"


def test_layernorm_program_keeps_only_what_is_read_again():
    spec = layernorm_stats_graph(24, 96, in_dtype="f32", out_dtype="f32", with_variance=True)
    plan = B.Plan(B.Graph.from_spec(spec), "auto")
    lines = [l.split() for l in plan.describe().splitlines() if l.strip().startswith("instr")]
    kept = [l for l in lines if "flags=vk" in l or "flags=sk" in l]
    # h, mean, the centred row, variance, rstd and the scaled values all pass through the accumulators:
    # the variance reduction squares on the fly, so nothing is written to a register
    assert len(kept) == 0 and any(l[2] == "rsumsq" for l in lines) and not any(l[2] in ("square", "cvt") for l in lines)
    head = [l for l in plan.describe().splitlines() if l.strip().startswith("program ")][0]
    assert "regs=1" in head and "sregs=0" in head       # x arrives in the accumulator, res is parked, the centred row reuses its slot


@pytest.mark.parametrize("seed", range(60))
def test_random_patterns_compile_to_correct_programs(seed):
    spec = random_row_pattern(seed, 11, 32, "f32", n_ops=6 + seed % 12)
    _compare(spec, seed=seed)


def test_patterns_that_are_not_row_local_are_refused():
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    # a column reduction whose result is read inside the pattern: values cross rows
    spec = GraphSpec("pattern_x", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("s", "reduce_sum", ("e",), {"axis": 0}), OpSpec("y", "div", ("e", "s"))],
                     [("y", "f32")])
    assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"
    # a column maximum: the fold kernel hands out sums only
    spec = GraphSpec("pattern_x", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("s", "reduce_max", ("e",), {"axis": 0})], [("s", "f32")])
    assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"
    # an output that is stretched itself would be written by several rows
    spec = GraphSpec("pattern_w", [TensorSpec("x", "f32", (4, 6, 16)), TensorSpec("m", "f32", (4, 1, 16))],
                     [OpSpec("a", "add", ("x", "m")), OpSpec("e", "exp", ("m",))], [("a", "f32"), ("e", "f32")])
    assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"
    # likewise a per-column value that is no sum over the rows (here beside one that is): it has no row to be stored to
    spec = GraphSpec("pattern_v", [TensorSpec("x", "f32", (40, 64)), TensorSpec("c", "f32", (64,))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("s", "reduce_sum", ("e",), {"axis": 0}), OpSpec("h", "scale", ("c",), {"value": 0.5})],
                     [("e", "f32"), ("s", "f32"), ("h", "f32")])
    assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"
    # a row too long for one workgroup's registers (1024 threads x 8 vectors at most) falls back without the run-time compiler
    spec = GraphSpec("pattern_z", [TensorSpec("x", "f32", (2, 1 << 17))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("y", "mul", ("e", "x"))], [("y", "f32")])
    with B.codegen(False):
        assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"
    # ... and 32768 floats fit 1024 threads (generated kernels) but not the interpreter's 256
    spec = GraphSpec("pattern_z", [TensorSpec("x", "f32", (2, 1 << 15))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("y", "mul", ("e", "x"))], [("y", "f32")])
    with B.codegen(False):
        assert B.Plan(B.Graph.from_spec(spec), "auto").info["scheme"] == "unfused"
    if B.codegen_available():
        info = B.Plan(B.Graph.from_spec(spec), "auto").info
        assert info["scheme"] == "lds" and info["block"][0] == 1024


@pytest.mark.parametrize("cols,dtype", [(1 << 17, "f32"), (50257, "f32"), (70000, "bf16")])
def test_rows_beyond_a_workgroups_registers_compile_to_passes_over_chunks(cols, dtype):
    """One pass over the row's chunks per row reduction (a row maximum that only shifts the exponentials of a row sum
    shares its pass with that sum), one more for the stores; the last chunk has its own extent."""
    if not B.codegen_available():
        pytest.skip("needs the run-time compiler")
    from workloads import softmax_graph
    for spec, reductions, shared in ((softmax_graph(3, cols, dtype), 2, 1),
                                     (layernorm_stats_graph(3, cols, in_dtype=dtype, out_dtype=dtype, with_variance=True), 2, 0),
                                     (silu_gate_graph(3, cols, dtype), 0, 0)):
        plan = B.Plan(B.Graph.from_spec(spec), "auto")
        info, src, listing = plan.info, plan.source(), plan.describe()
        assert info["pattern"] == "row_generated" and "chunks" in info["kernel"] and info["n_kernels"] == 1
        line = listing[listing.index("  chunks "):].splitlines()[0].split()
        chunks, width, kept = int(line[1]), int(line[3]), (int(line[7]) if "kept" in line else 0)
        assert (chunks - 1) * width < cols <= chunks * width and width == info["lanes_per_row"] * info["vecs_per_lane"] * (8 if "<v8" in info["kernel"] else 4 if "<v4" in info["kernel"] else 1)
        assert kept == 0 or reductions > 0                      # keeping chunks in registers only pays when a later pass reads them
        passes = reductions + 1 - shared
        looped, tail_apart = kept < chunks - 1, kept < chunks    # what is not kept: whole chunks by a loop, the last chunk by itself
        assert src.count("for (uint32_t chunk = ") == (passes if looped else 0) and src.count("Row::finish<") == reductions
        # (the loads that a shared first pass issues up front name the last chunk once more when it is kept too)
        assert src.count(f"TailRow row(fs_block, 0, {(chunks - 1) * width}u)") == passes + (1 if shared and kept == chunks else 0)
        # kept chunks are unpacked anew in every later pass; a shared first pass loads all of them up front and then
        # unpacks them one by one as well
        unpackings = passes - 1 + (1 if shared else 0)
        assert src.count(".forget_contents();") == kept * unpackings * sum(1 for t in spec.inputs if len(t.dims) == 2 and t.dims[-1] == cols)
        assert src.count("m_run = m_new;") == (kept + (1 if looped else 0) + (1 if tail_apart else 0)) * shared
        # every full-shaped output is stored in the last pass only, once per piece of source that handles a chunk
        ref = O.evaluate(spec, make_inputs(spec, seed=4))
        n_full_out = sum(1 for name, _ in spec.outputs if ref[name].shape[-1] == cols)
        pieces = kept + (1 if looped else 0) + (1 if tail_apart else 0)
        assert src.count("row.store<") == pieces * n_full_out and src.count("row.store_scalar<") == len(spec.outputs) - n_full_out
        got, _ = emulate(listing, spec, make_inputs(spec, seed=4), (3, cols))
        for name, dt in spec.outputs:
            r = ref[name].reshape(got[name].shape)
            assert O.max_rel_err(got[name], r, O.rms(r)) < 2e-5, (spec.name, name)
