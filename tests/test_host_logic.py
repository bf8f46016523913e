"""Host-side logic of the library, no GPU needed: exports, descriptor validation,
pattern matching, candidate enumeration, plan queries, error codes."""
import ctypes
import os
import re

import pytest

from paper_2009_10924_amd import binding as B
from workloads import (FULL_CONFIGS, add_bias_layernorm_graph, attention_scores_graph, bias_gelu_dbias_graph,
                       bias_gelu_graph, softmax_graph, transpose_chain_graph, transpose_graph)
from workloads.graphs import GraphSpec, OpSpec, TensorSpec

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "fusion_stitching.h")).read()
    declared = set(re.findall(r"\b(fs_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert b"gfx950" in lib.fs_version()


def test_enum_values_match_header():
    header = open(os.path.join(ROOT, "include", "fusion_stitching.h")).read()
    for name, val in [("FS_ADD", 0), ("FS_MAX", 4), ("FS_SCALE", 5), ("FS_ADD_SCALAR", 6), ("FS_SQUARE", 7),
                      ("FS_EXP", 8), ("FS_RSQRT", 9), ("FS_TANH", 10), ("FS_GELU_TANH", 11),
                      ("FS_GELU_TANH_GRAD", 12), ("FS_BROADCAST", 13), ("FS_REDUCE_SUM", 14),
                      ("FS_REDUCE_MAX", 15), ("FS_REDUCE_MEAN", 16), ("FS_TRANSPOSE", 17), ("FS_CONVERT", 18)]:
        assert re.search(rf"\b{name} = {val}\b", header), name
    assert B.OPCODE["reduce_mean"] == 16 and B.OPCODE["convert"] == 18


def test_header_is_plain_c_and_struct_layout_matches(tmp_path):
    # the header must compile as C; sizes / offsets of the structs the binding mirrors must agree
    src = tmp_path / "layout.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "fusion_stitching.h"\n'
        'int main(void){printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu\\n", sizeof(fs_plan_info), offsetof(fs_plan_info, workspace_bytes),'
        ' offsetof(fs_plan_info, predicted_us), offsetof(fs_plan_info, kernel), sizeof(fs_plan_opts), sizeof(fs_attr_dims),'
        ' sizeof(fs_pack_info), offsetof(fs_pack_info, bytes_min), offsetof(fs_pack_info, predicted_separate_us));return 0;}\n')
    exe = tmp_path / "layout"
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    got = [int(v) for v in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    I = B.fs_plan_info
    assert got == [ctypes.sizeof(I), I.workspace_bytes.offset, I.predicted_us.offset, I.kernel.offset,
                   ctypes.sizeof(B.fs_plan_opts), ctypes.sizeof(B.fs_attr_dims),
                   ctypes.sizeof(B.fs_pack_info), B.fs_pack_info.bytes_min.offset, B.fs_pack_info.predicted_separate_us.offset]


@pytest.mark.parametrize("cfg", ["C1", "C2", "C3", "C4", "C5"])
def test_full_configs_match_a_stitched_pattern(cfg):
    spec = FULL_CONFIGS[cfg]()
    g = B.Graph.from_spec(spec)
    plan = B.Plan(g, "auto")
    info = plan.info
    expect = {"C1": ("softmax", 65536), "C2": ("layernorm", 62923776), "C3": ("softmax", 25174016),
              "C4": ("bias_gelu_dbias", 302008320), "C5": ("transpose_chain", 201326640)}[cfg]
    assert info["pattern"] == expect[0]
    assert info["bytes_min"] == expect[1]          # each input read once + each output written once
    # one launch, or two when the column sums are folded by a second tiny launch
    assert info["n_kernels"] == 1 or (cfg == "C4" and info["n_kernels"] == 2 and info["kernel"].endswith("fold>"))
    assert info["predicted_us"] > 0
    cands = plan.candidates()
    assert len(cands) == info["n_candidates"] >= 1
    assert min(c["predicted_us"] for c in cands) == info["predicted_us"]
    # the per-op plan launches one kernel per op (column reduction: partials + fold)
    unf = B.Plan(g, "unfused").info
    n_ops = len(spec.ops)
    assert unf["n_kernels"] == n_ops + (1 if cfg == "C4" else 0)
    assert unf["bytes_moved_model"] > 3 * info["bytes_min"]
    assert unf["scheme"] == "unfused"


def test_scheme_selection_and_locality():
    g = B.Graph.from_spec(add_bias_layernorm_graph(64, 768))
    assert B.Plan(g, "wave").info["scheme"] == "wave"
    assert B.Plan(g, "lds").info["scheme"] == "lds"
    with pytest.raises(B.FsError) as e:
        B.Plan(g, "global")
    assert e.value.code == -6                       # FS_ERR_LOCALITY
    # a row too long for one wavefront's registers cannot use the wave scheme
    g_long = B.Graph.from_spec(softmax_graph(4, 4096, "f32"))
    with pytest.raises(B.FsError) as e:
        B.Plan(g_long, "wave")
    assert e.value.code == -6
    assert B.Plan(g_long, "lds").info["scheme"] == "lds"
    # forcing a launch shape
    p = B.Plan(g, "wave", vecs_per_lane=6)
    assert p.info["vecs_per_lane"] == 6 and p.info["lanes_per_row"] == 32
    with pytest.raises(B.FsError):
        B.Plan(g, "wave", vecs_per_lane=5)
    p2 = B.Plan(g, "wave", candidate=0)
    assert p2.info["candidate"] == 0


def test_unsupported_pattern_and_auto_fallback():
    # exp(transpose(x)): valid graph, but values move between rows, so no stitched kernel
    spec = GraphSpec("custom", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("t", "transpose", ("x",), {"perm": (1, 0)}), OpSpec("y", "exp", ("t",))], [("y", "f32")])
    g = B.Graph.from_spec(spec)
    with pytest.raises(B.FsError) as e:
        B.Plan(g, "wave")
    assert e.value.code == -5                       # FS_ERR_UNSUPPORTED_PATTERN
    info = B.Plan(g, "auto").info
    assert info["scheme"] == "unfused" and info["n_kernels"] == 2
    # exp(x) * x has no hand-written family, but is row-local: one interpreted kernel
    spec = GraphSpec("custom", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("y", "mul", ("e", "x"))], [("y", "f32")])
    info = B.Plan(B.Graph.from_spec(spec), "auto").info
    assert info["pattern"] in ("row_program", "row_generated") and info["n_kernels"] == 1 and info["workspace_bytes"] == 0
    assert ",I3," in info["kernel"]                 # exp (x arrives in the accumulator), mul by x, store
    # ragged softmax still gets a stitched (block-per-row) kernel
    with B.codegen(False):
        info = B.Plan(B.Graph.from_spec(softmax_graph(5, 37, "f32")), "auto").info
    assert info["pattern"] == "softmax" and info["scheme"] == "lds"
    if B.codegen_available():       # with the run-time compiler, a kernel generated for the row length takes over
        info = B.Plan(B.Graph.from_spec(softmax_graph(5, 37, "f32")), "auto").info
        assert info["pattern"] == "row_generated" and info["n_candidates"] > 1


def test_commuted_operands_still_match():
    # bias + x instead of x + bias, gamma * n instead of n * gamma
    spec = add_bias_layernorm_graph(16, 256)
    ops = []
    for op in spec.ops:
        if op.out in ("h", "g", "o", "h0"):
            ops.append(OpSpec(op.out, op.opcode, tuple(reversed(op.inputs)), op.attr))
        else:
            ops.append(op)
    info = B.Plan(B.Graph.from_spec(GraphSpec("add_bias_layernorm_commuted", spec.inputs, ops, spec.outputs)), "auto").info
    assert info["pattern"] == "layernorm"


def test_descriptor_validation_errors(lib):
    g = B.Graph()
    x = g.input("f32", (4, 8))
    y = g.input("f32", (3, 8))
    with pytest.raises(B.FsError) as e:
        g.op("add", [x, y])
    assert e.value.code == -2 and "broadcast" in e.value.text
    with pytest.raises(B.FsError) as e:
        g.op("add", [x, 99])
    assert e.value.code == -4                       # operand does not precede the op
    with pytest.raises(B.FsError) as e:
        g.op("reduce_sum", [x], axis=2)
    assert e.value.code == -2
    with pytest.raises(B.FsError) as e:
        g.op("transpose", [x], perm=(0, 0))
    assert e.value.code == -2
    with pytest.raises(B.FsError) as e:
        g.input("f32", (0, 8))
    assert e.value.code == -2 and "empty" in e.value.text
    with pytest.raises(B.FsError):
        g.input("f32", (1, 2, 3, 4, 5))
    with pytest.raises(B.FsError) as e:
        g.input("f32", (1 << 16, 1 << 16))
    assert e.value.code == -2
    i = g.input("i32", (4, 8))
    with pytest.raises(B.FsError) as e:
        g.op("exp", [i])
    assert e.value.code == -3
    with pytest.raises(B.FsError):
        g.finalize()                                # no output yet
    e1 = g.op("exp", [x])
    g.op("square", [x])                             # dead result
    g.output(e1, "f32")
    with pytest.raises(B.FsError) as e:
        g.finalize()
    assert "neither consumed nor an output" in e.value.text
    with pytest.raises(B.FsError):
        g.output(e1, "f32")                         # twice
    with pytest.raises(B.FsError):
        B.Plan(g, "auto")                           # not finalized
    # null handles never crash
    assert lib.fs_graph_finalize(None) == -1
    assert lib.fs_plan_query(None, None) == -1
    assert lib.fs_execute(None, None, None, None, 0, None) == -1
    lib.fs_graph_destroy(None)
    lib.fs_plan_destroy(None)


def test_unfused_plan_shapes():
    # transpose that moves the innermost axis goes through the LDS tile kernel
    info = B.Plan(B.Graph.from_spec(transpose_graph((6, 40, 70), (2, 0, 1), "f16")), "unfused").info
    assert info["kernel"] == "transpose_tile" and info["n_kernels"] == 1
    info = B.Plan(B.Graph.from_spec(transpose_graph((6, 40, 70), (1, 0, 2), "f32")), "unfused").info
    assert info["kernel"] == "transpose_rows"
    # workspace of the per-op softmax: m, s, e, z live, buffers reused after their last reader
    info = B.Plan(B.Graph.from_spec(softmax_graph(64, 128)), "unfused").info
    assert info["n_kernels"] == 5
    assert 0 < info["workspace_bytes"] <= 2 * 64 * 128 * 4 + 2 * 256
    assert info["bytes_moved_model"] == 263168      # 4.0 x bytes_min with float32 intermediates
    info = B.Plan(B.Graph.from_spec(bias_gelu_graph(32, 64)), "auto").info
    assert info["pattern"] == "bias_gelu" and info["scheme"] == "local"
    info = B.Plan(B.Graph.from_spec(attention_scores_graph(2, 3, 8, 64)), "auto").info
    assert info["pattern"] == "softmax"
    info = B.Plan(B.Graph.from_spec(transpose_chain_graph(2, 9, 3, 64)), "lds").info
    assert info["pattern"] == "transpose_chain" and info["lds_bytes"] > 0
    info = B.Plan(B.Graph.from_spec(bias_gelu_dbias_graph(100, 520)), "global").info
    assert info["workspace_bytes"] > 0 and info["scheme"] == "global"


def test_pack_creation_and_errors(lib):
    from workloads.graphs import add_bias_layernorm_graph, rmsnorm_graph, softmax_backward_graph
    specs = [softmax_graph(64, 128, "f32"), add_bias_layernorm_graph(100, 768), rmsnorm_graph(50, 4096),
             softmax_backward_graph(77, 256, "f16"), bias_gelu_graph(33, 3072)]
    before = B.codegen_enable(False)          # the fixed packed kernel and its closed set of member forms
    try:
        _fixed_pack_checks(lib, specs)
    finally:
        B.codegen_enable(before)


def _fixed_pack_checks(lib, specs):
    plans = [B.Plan(B.Graph.from_spec(s), "auto") for s in specs]
    info = B.Pack(plans).info
    assert info["generated"] == 0
    # 8 rows / workgroup, 4 rows / workgroup, then one workgroup per row (rows longer than 64 lanes x 4 vectors), 8 rows, per row
    assert info["grid"] == 8 + 25 + 50 + 10 + 33 and info["block"] == 256
    assert info["n_members"] == 5 and info["n_kernels"] == 1
    assert info["n_inputs"] == 1 + 5 + 2 + 2 + 2 and info["n_outputs"] == 5
    assert info["bytes_min"] == sum(p.info["bytes_min"] for p in plans)
    assert info["predicted_us"] < info["predicted_separate_us"]
    # 33 members need two launches
    assert B.Pack([plans[0]] * 33).info["n_kernels"] == 2
    with pytest.raises(B.FsError) as e:       # masked softmax has no packed form
        B.Pack([plans[0], B.Plan(B.Graph.from_spec(attention_scores_graph(2, 2, 16, 16)), "auto")])
    assert e.value.code == -5 and "plan 1" in e.value.text
    with pytest.raises(B.FsError) as e:       # per-op plans carry no pattern
        B.Pack([B.Plan(B.Graph.from_spec(softmax_graph(8, 64)), "unfused")])
    assert e.value.code == -5
    with pytest.raises(B.FsError) as e:       # row too long for one workgroup
        B.Pack([B.Plan(B.Graph.from_spec(softmax_graph(4, 16384, "f32")), "auto")])
    assert e.value.code == -6
    with pytest.raises(B.FsError) as e:
        B.Pack([])
    assert e.value.code == -1
    with pytest.raises(B.FsError):
        B.Pack([plans[0]] * (B.FS_PACK_MAX_MEMBERS + 1))
    assert lib.fs_pack_query(None, None) == -1
    assert lib.fs_pack_execute(None, None, None, None) == -1
    lib.fs_pack_destroy(None)


def test_generated_pack_takes_any_row_local_member(lib):
    """With the run-time compiler a pack is a kernel generated for exactly its members: masked softmax, patterns with
    several outputs, folded transposes and patterns of no family at all can join; column reductions and per-op plans
    cannot."""
    if not B.codegen_available():
        pytest.skip("needs the run-time compiler")
    from workloads import bias_head_split_graph, layernorm_stats_graph, random_row_pattern, silu_gate_graph
    from workloads.graphs import add_bias_layernorm_graph
    specs = [softmax_graph(64, 128, "f32"), attention_scores_graph(2, 2, 16, 64), layernorm_stats_graph(30, 96, with_variance=True),
             bias_head_split_graph(2, 5, 3, 16, "bf16"), silu_gate_graph(9, 50, "f16"), random_row_pattern(5, 20, 64, "f32", n_ops=9),
             add_bias_layernorm_graph(100, 768)]
    plans = [B.Plan(B.Graph.from_spec(s), "auto") for s in specs]
    pack = B.Pack(plans)
    info = pack.info
    assert info["generated"] == 1 and info["n_kernels"] == 1 and info["n_members"] == len(specs)
    assert info["n_inputs"] == sum(len(s.inputs) for s in specs) and info["n_outputs"] == sum(len(s.outputs) for s in specs)
    assert info["grid"] >= len(specs) and 0 < info["vgprs"] <= 256
    assert B.Pack([plans[0]] * 33).info["n_kernels"] == 2
    with pytest.raises(B.FsError) as e:       # a column reduction needs a fold launch of its own
        B.Pack([plans[0], B.Plan(B.Graph.from_spec(bias_gelu_dbias_graph(100, 520)), "auto")])
    assert e.value.code == -5
    with pytest.raises(B.FsError) as e:       # per-op plans carry no pattern
        B.Pack([B.Plan(B.Graph.from_spec(softmax_graph(8, 64)), "unfused")])
    assert e.value.code == -5


def test_zero_initialised_plan_opts_ask_for_nothing(lib):
    # the C idiom `fs_plan_opts o = {0}; o.block_threads = 256;` must leave the choice to the evaluator:
    # `candidate` counts from 1, zero means "choose"
    import ctypes as C
    spec = FULL_CONFIGS["C2"]()
    g = B.Graph.from_spec(spec)
    auto = B.Plan(g, "auto").info
    h = C.c_void_p()
    opts = B.fs_plan_opts(0, 0, 0, 0)
    assert lib.fs_plan_create(g.handle, B.SCHEME["auto"], C.byref(opts), C.byref(h)) == 0
    info = B.fs_plan_info()
    assert lib.fs_plan_query(h, C.byref(info)) == 0
    assert info.candidate == auto["candidate"] and info.kernel.decode() == auto["kernel"]
    lib.fs_plan_destroy(h)
    # k > 0 takes entry k - 1, whatever the other fields say
    for k in (1, auto["n_candidates"]):
        opts = B.fs_plan_opts(k, 0, 0, 0)
        assert lib.fs_plan_create(g.handle, B.SCHEME["auto"], C.byref(opts), C.byref(h)) == 0
        assert lib.fs_plan_query(h, C.byref(info)) == 0
        assert info.candidate == k - 1
        lib.fs_plan_destroy(h)
    opts = B.fs_plan_opts(auto["n_candidates"] + 1, 0, 0, 0)
    assert lib.fs_plan_create(g.handle, B.SCHEME["auto"], C.byref(opts), C.byref(h)) == -1


def test_static_scratch_entry_point_checks_before_touching_the_gpu(lib):
    # size and pointer checks come before any HIP call, so they can be exercised without a GPU
    import ctypes as C
    spec = FULL_CONFIGS["C4"]()
    g = B.Graph.from_spec(spec)
    per_op = B.Plan(g, "unfused")
    assert per_op.info["workspace_bytes"] > B.FS_STATIC_SCRATCH_BYTES
    with pytest.raises(B.FsError) as e:
        per_op.execute_static_ptrs([256] * len(spec.inputs), [256] * len(spec.outputs), 0)
    assert e.value.code == -7 and "static array" in e.value.text
    stitched = B.Plan(g, "auto")
    assert 0 < stitched.info["workspace_bytes"] <= B.FS_STATIC_SCRATCH_BYTES
    with pytest.raises(B.FsError) as e:
        stitched.execute_static_ptrs([256, 8, 256], [256] * len(spec.outputs), 0)
    assert e.value.code == -8
    with pytest.raises(B.FsError) as e:
        stitched.execute_static_ptrs([256, 0, 256], [256] * len(spec.outputs), 0)
    assert e.value.code == -1
    # the header's constant and the binding's agree
    header = open(os.path.join(ROOT, "include", "fusion_stitching.h")).read()
    assert "#define FS_STATIC_SCRATCH_BYTES (4u << 20)" in header and B.FS_STATIC_SCRATCH_BYTES == 4 << 20


def test_stream_probe_checks_its_arguments_before_touching_the_gpu(lib):
    # every refusal below is decided on the host, before any launch
    def code(**kw):
        a = dict(dst=256, src=256, stream_bytes=4096, reads=2, writes=1, vecs=2, pitch=0)
        a.update(kw)
        try:
            B.bind_probe(a["dst"], a["src"], a["stream_bytes"], a["reads"], a["writes"], a["vecs"], 0, a["pitch"])()
        except B.FsError as e:
            return e.code
        return 0
    assert code(dst=0) == -1 and code(src=0) == -1                       # null pointers (a source is needed when anything is read)
    assert code(reads=5) == -1 and code(writes=3) == -1 and code(reads=0, writes=0) == -1
    assert code(vecs=3) == -1 and code(reads=-1) == -1
    assert code(dst=264) == -8 and code(stream_bytes=4100) == -8 and code(pitch=4104) == -8   # 16-byte rule
    assert code(pitch=2048) == -2                                         # FS_ERR_SHAPE: the streams would overlap
    assert code(stream_bytes=0) == 0                                      # nothing to move: no launch, no error
