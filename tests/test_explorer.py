"""Fusion explorer (paper Section 5), checked on the CPU.

The library's search is compared with a plain Python restatement of the paper's procedure
(oracle/explorer.py) that gets pattern scores from the library's delta-evaluator through a callback, with an
exhaustive search on tiny graphs, and with structural invariants (patterns disjoint, covering, free of
cyclic dependences).  Nothing here launches a kernel."""
import numpy as np
import pytest

from oracle import explorer as X
from paper_2009_10924_amd import binding as B
from workloads import (FULL_CONFIGS, NEXT_CONFIGS, add_bias_layernorm_graph, attention_scores_graph, bias_gelu_dbias_graph,
                       layernorm_backward_graph, layernorm_stats_graph, random_multi_pattern, random_row_pattern,
                       softmax_graph, transformer_block_graph, transpose_chain_graph)
from workloads.graphs import GraphSpec, OpSpec, TensorSpec


def _score_fn(graph):
    def score(ops):
        f, f_opt, code = B.explore_score_ex(graph, list(ops))
        return (0 if code == 0 else ("unsupported" if code == -5 else code)), f, f_opt
    return score


def _explore_both(spec, **opts):
    g = B.Graph.from_spec(spec)
    prog = B.Program(g, **opts)
    view = X.GraphView(spec)
    cand, plans = X.explore(view, _score_fn(g), top_k=opts.get("top_k", 0) or 3, beam_width=opts.get("beam_width", 0) or 3)
    return prog, view, cand, plans


def _multi(prog):
    return sorted(tuple(p["ops"]) for p in prog.patterns() if len(p["ops"]) > 1)


SPECS = {
    "transformer_block_small": lambda: transformer_block_graph(2, 16, 2, 8, 64, "bf16"),
    "transformer_block": lambda: transformer_block_graph(32, 128, 12, 64, 3072, "bf16"),
    "softmax": lambda: softmax_graph(64, 128, "f32"),
    "layernorm": lambda: add_bias_layernorm_graph(128, 768),
    "attention": lambda: attention_scores_graph(2, 3, 16, 64),
    "gelu_dbias": lambda: bias_gelu_dbias_graph(256, 512),
    "transpose_chain": lambda: transpose_chain_graph(2, 16, 4, 64),
    "layernorm_backward": lambda: layernorm_backward_graph(64, 256, "f32"),
    "layernorm_stats": lambda: layernorm_stats_graph(64, 256, with_variance=True),
}
SPECS.update({f"multi{s}": (lambda s=s: random_multi_pattern(s)) for s in range(16)})
# graphs with matrix products taken out and declared (patterns may not span them)
SPECS.update({f"multi_outside{s}": (lambda s=s: random_multi_pattern(s, rows=64, cols=128, segments=2 + s % 3, external_links=True,
                                                                    column_sums=s % 2)) for s in range(8)})
SPECS["block_forward"] = lambda: transformer_block_graph(2, 16, 2, 8, 64, "bf16")
SPECS["block_forward_biases"] = lambda: transformer_block_graph(2, 16, 2, 8, 64, "bf16", projection_bias=True)
SPECS["block_backward"] = lambda: __import__("workloads").transformer_block_backward_graph(2, 16, 2, 8, 64, "bf16")
SPECS.update({f"multi_sums{s}": (lambda s=s: random_multi_pattern(s, rows=64, cols=128, segments=2 + s % 3, column_sums=1 + s % 2)) for s in range(8)})
SPECS.update({f"multi_big{s}": (lambda s=s: random_multi_pattern(100 + s, rows=512, cols=1024, segments=4)) for s in range(4)})


def test_patterns_that_wait_for_each_other_are_not_a_plan():
    """{a, d} and {b, c} with a -> b and c -> d: each is convex, together they have no order of execution."""
    from workloads.graphs import GraphSpec, OpSpec, TensorSpec
    spec = GraphSpec("pattern_circle", [TensorSpec("x", "f32", (8, 16)), TensorSpec("y", "f32", (8, 16))],
                     [OpSpec("a", "exp", ("x",)), OpSpec("b", "tanh", ("a",)), OpSpec("c", "tanh", ("y",)), OpSpec("d", "exp", ("c",))],
                     [("a", "f32"), ("b", "f32"), ("c", "f32"), ("d", "f32")])
    view = X.GraphView(spec)
    assert X.plan_is_acyclic(view, [(0, 1), (2, 3)]) and X.plan_is_acyclic(view, [(0, 2), (1, 3)]) and X.plan_is_acyclic(view, [(0, 3)])
    assert not X.plan_is_acyclic(view, [(0, 3), (1, 2)])
    # the library never returns such a plan: whatever it merges, the steps come back in an order that runs
    prog = B.Program(B.Graph.from_spec(spec))
    done = set()
    for st in prog.patterns():
        assert all(p in done or p in st["ops"] for o in st["ops"] for p in view.producers[o])
        done |= set(st["ops"])


@pytest.mark.parametrize("name", sorted(SPECS))
def test_library_plan_is_one_of_the_oracle_beam_plans(name):
    spec = SPECS[name]()
    prog, view, cand, plans = _explore_both(spec)
    g = B.Graph.from_spec(spec)
    score = _score_fn(g)

    def finished(plan):       # the beam plan after remote fusion: its multi-op groups and its total score
        groups, gain = X.remote_fusion(plan[0], len(spec.ops), score, view)
        return sorted(p for p in groups if len(p) > 1), plan[1] + gain
    got = _multi(prog)
    beam = [finished(p) for p in plans]
    assert got in [b[0] for b in beam], f"{name}: library chose {got}, the oracle's beam holds {beam}"
    f_oracle = beam[[b[0] for b in beam].index(got)][1]
    assert abs(prog.info["f_total_us"] - f_oracle) <= 1e-9 * max(1.0, abs(f_oracle))
    # with a beam of one there is no final choice left: the plans must be identical
    prog1, _, _, plans1 = _explore_both(spec, beam_width=1)
    want1 = finished(plans1[0])
    assert _multi(prog1) == want1[0]
    assert abs(prog1.info["f_total_us"] - want1[1]) <= 1e-9 * max(1.0, abs(want1[1]))
    # and without remote fusion the beam plans themselves
    prog2 = B.Program(g, no_remote_fusion=True)
    assert _multi(prog2) in [sorted(p) for p, _ in plans]


@pytest.mark.parametrize("name", sorted(SPECS))
def test_plan_structure(name):
    spec = SPECS[name]()
    g = B.Graph.from_spec(spec)
    prog = B.Program(g)
    view = X.GraphView(spec)
    steps = prog.patterns()
    seen = set()
    done = set()
    for st in steps:
        ops = st["ops"]
        assert ops == sorted(ops) and not (seen & set(ops))
        seen |= set(ops)
        inside = set(ops)
        # convex: nothing outside lies between two members
        below = set().union(*(view.after[o] for o in ops)) - inside
        assert not any(view.after[x] & inside for x in below), f"{name}: pattern {ops} has a cyclic dependence"
        # nothing in a pattern waits for another member through an external computation, and what it waits for has run
        for o in ops:
            assert not (set(view.waiting[o]) & inside), f"{name}: pattern {ops} spans an external computation"
        for p in range(view.n):
            if set(view.waiting[p]) & inside:
                assert p in done, f"{name}: {ops} runs before op {p}, whose result it needs through an external computation"
        # execution order: every producer outside the pattern has run
        for o in ops:
            assert all(p in done or p in inside for p in view.producers[o]), f"{name}: {ops} runs before its producers"
        done |= inside
        if len(ops) > 1:
            assert st["f_us"] > 0 and st["info"]["scheme"] != "unfused"
            assert abs(st["f_us"] - B.explore_score(g, ops)) < 1e-9
    assert seen == set(range(len(spec.ops)))
    info = prog.info
    assert info["n_patterns"] + info["n_single_ops"] == len(steps)
    assert info["n_kernels"] <= len(spec.ops) and info["predicted_us"] > 0
    assert abs(info["f_total_us"] - sum(s["f_us"] for s in steps)) < 1e-6


def test_transformer_block_plan_is_the_hand_partition():
    """With the compiled-in kernels alone the explorer finds the partition one would write by hand (the three head-split
    moves of q, k and v, which share a row space, go out as one interpreted row program)."""
    spec = transformer_block_graph(32, 128, 12, 64, 3072, "bf16")
    with B.codegen(False):
        prog = B.Program(B.Graph.from_spec(spec))
    steps = prog.patterns()
    names = sorted((s["info"]["pattern"], len(s["ops"])) for s in steps)
    assert names == sorted([("transpose", 1), ("row_program", 3), ("softmax", 7), ("layernorm", 12), ("bias_gelu", 2), ("layernorm", 12)])
    assert prog.info["n_kernels"] == 6 and prog.info["workspace_bytes"] == 0   # every tensor between patterns is a graph output
    # the second LayerNorm reads what the first one stored
    order = [tuple(s["ops"]) for s in steps]
    assert order.index(tuple(range(11, 23))) < order.index(tuple(range(25, 37)))


def test_matrix_products_between_patterns_keep_them_apart():
    """The block's graph says which input each matrix product computes from which outputs.  Without that knowledge
    the two LayerNorm neighbourhoods, the second of which reads what the first stored, look like ONE 24-op pattern
    (and a generated kernel can run it); in the block they are five matrix-product-separated stages apart, and the
    plan is the hand partition, run stage by stage."""
    spec = transformer_block_graph(32, 128, 12, 64, 3072, "bf16")
    g = B.Graph.from_spec(spec)
    prog = B.Program(g)
    steps = prog.patterns()
    assert sorted(o for s in steps for o in s["ops"]) == list(range(len(spec.ops)))
    assert max(len(s["ops"]) for s in steps) == 12 and prog.info["n_kernels"] == 6 and prog.info["n_stages"] == 6
    text = prog.describe()
    stages = [int(l.split("stage=")[1].split()[0]) for l in text.splitlines() if l.startswith("step ")]
    assert stages == sorted(stages) == [0, 1, 2, 3, 4, 5]
    with pytest.raises(B.FsError) as e:        # no single plan can run a graph that waits for outside work in the middle
        B.Plan(g, "auto")
    assert e.value.code == -5 and "external" in e.value.text
    if B.codegen_available():
        free = B.Program(B.Graph.from_spec(transformer_block_graph(32, 128, 12, 64, 3072, "bf16", matmul_dependences=False)))
        big = max(free.patterns(), key=lambda s: len(s["ops"]))
        assert tuple(big["ops"]) == tuple(range(11, 23)) + tuple(range(25, 37)) and free.info["n_stages"] == 1
        assert free.info["n_kernels"] < prog.info["n_kernels"]


def test_a_stack_of_blocks_is_explored_block_by_block():
    """Six blocks, 222 ops: six launches per block, one stage per stretch between matrix products, found in seconds."""
    import time
    from workloads import transformer_stack_graph
    spec = transformer_stack_graph(6, 2, 16, 2, 8, 64, "bf16")
    assert len(spec.ops) == 6 * 37
    g = B.Graph.from_spec(spec)
    t0 = time.perf_counter()
    prog = B.Program(g)
    assert time.perf_counter() - t0 < 30.0
    assert prog.info["n_kernels"] == 36 and prog.info["n_stages"] == 36
    view = X.GraphView(spec)
    done = set()
    for st in prog.patterns():
        inside = set(st["ops"])
        assert all(p in done or p in inside for o in st["ops"] for p in view.producers[o])
        assert not any(set(view.waiting[o]) & inside for o in st["ops"])
        assert all(p in done for p in range(view.n) if set(view.waiting[p]) & inside)
        done |= inside
    assert done == set(range(len(spec.ops)))


def test_external_dependences_are_checked_when_declared():
    lib = B.load()
    g = B.Graph()
    x = g.input("f32", (8, 16))
    y = g.input("f32", (8, 16))
    e = g.op("exp", [x])
    assert lib.fs_graph_external(g.handle, x, y) == -1          # the source must be an op's result
    assert lib.fs_graph_external(g.handle, e, e) == -1          # the target must be a graph input
    assert lib.fs_graph_external(g.handle, e, y) == 0
    t = g.op("tanh", [y])
    assert lib.fs_graph_external(g.handle, e, y) == -1          # too late: something reads the input already
    g.output(t, "f32")
    assert lib.fs_graph_finalize(g.handle) == -1                # what an external computation reads must be an output
    assert "must be a graph output" in lib.fs_last_error().decode()
    g.output(e, "f32")
    g.finalize()
    prog = B.Program(g)
    assert prog.info["n_stages"] == 2 and prog.info["n_kernels"] == 2


def test_backward_block_folds_its_column_sums_in_one_launch_at_the_end():
    """Bias and gain gradients are sums over all rows that nothing in the graph reads: their fold launches move behind
    the last step and run as one; the two bias gradients whose operands are graph inputs share one pattern."""
    if not B.codegen_available():
        pytest.skip("column sums inside patterns need the run-time compiler")
    from workloads import transformer_block_backward_graph
    spec = transformer_block_backward_graph(3, 40, 4, 32, 256, "bf16")
    g = B.Graph.from_spec(spec)
    prog, apart = B.Program(g), B.Program(g, no_joint_folds=True)
    assert prog.info["n_joint_folds"] >= 3 and apart.info["n_joint_folds"] == 0
    assert prog.info["n_kernels"] < apart.info["n_kernels"]
    assert prog.info["predicted_us"] < apart.info["predicted_us"]
    assert [s["ops"] for s in prog.patterns()] == [s["ops"] for s in apart.patterns()]      # the patterns are the same
    sums = [s for s in prog.patterns() if s["info"]["kernel"].endswith("+colfold")]
    assert len(sums) >= 2 and all(s["info"]["n_kernels"] >= 2 for s in sums)                  # a plan alone keeps its folds


def test_program_listing_names_steps_buffers_and_joint_folds():
    from workloads import transformer_block_backward_graph
    spec = transformer_block_backward_graph(3, 40, 4, 32, 256, "bf16")
    prog = B.Program(B.Graph.from_spec(spec))
    text = prog.describe()
    lines = text.splitlines()
    steps = [l for l in lines if l.startswith("step ")]
    assert lines[0].startswith("program steps=") and len(steps) == len(prog.patterns())
    for l, st in zip(steps, prog.patterns()):
        assert f"ops={','.join(map(str, st['ops']))} " in l and f"kernel={st['info']['kernel']} " in l
    # every graph input and output appears where a step binds it; what crosses steps lives in the workspace
    assert all(f" in{k}" in text for k in range(len(spec.inputs))) and all(f" out{k}" in text for k in range(len(spec.outputs)))
    issued = [l for l in lines if l.startswith("step ") or l.startswith("pack ")]
    assert sum(int(l.split("launches=")[1].split()[0]) for l in issued) + len([l for l in lines if l.startswith("joint_fold ")]) == prog.info["n_kernels"]
    if prog.info["n_joint_folds"]:
        assert sum(int(l.split("folds=")[1].split()[0]) for l in lines if l.startswith("joint_fold ")) == prog.info["n_joint_folds"]
    lib = B.load()
    assert lib.fs_program_describe(None, None, 0) == -1
    import ctypes
    small = ctypes.create_string_buffer(16)
    assert lib.fs_program_describe(prog.handle, small, 16) == len(text) + 1 and small.value.decode() == text[:15]


def test_independent_launch_bound_patterns_share_one_packed_launch():
    from workloads import independent_tiny_patterns_graph
    spec = independent_tiny_patterns_graph()
    g = B.Graph.from_spec(spec)
    prog = B.Program(g)
    steps = prog.patterns()
    assert prog.info["n_patterns"] == 8 and prog.info["n_packs"] == 1 and prog.info["n_kernels"] == 1
    assert all(s["pack"] == 0 for s in steps)
    apart = B.Program(g, no_packing=True)
    assert apart.info["n_packs"] == 0 and apart.info["n_kernels"] == 8
    assert prog.info["predicted_us"] < apart.info["predicted_us"]


@pytest.mark.parametrize("seed", range(24))
def test_explorer_against_exhaustive_search_on_tiny_graphs(seed):
    if seed % 2:
        spec = random_multi_pattern(200 + seed, rows=8, cols=16, segments=2, seg_ops=(2, 3))
    else:
        spec = random_row_pattern(300 + seed, 8, 16, "f32", n_ops=5 + seed % 4)
    if len(spec.ops) > 10:
        pytest.skip("too many ops for the exhaustive search")
    g = B.Graph.from_spec(spec)
    best = X.brute_force_best(X.GraphView(spec), _score_fn(g))
    got = B.Program(g).info["f_total_us"]
    assert got <= best + 1e-9
    assert got >= 0.9 * best - 1e-9, f"explorer found {got:.3f} us of gain, exhaustive search {best:.3f}"
    print(f"seed {seed}: {len(spec.ops)} ops, explorer {got:.3f} us, optimum {best:.3f} us")


def test_delta_evaluator_terms():
    # f = reduced memory time + reduced launches - penalty: for a pure element-wise chain of n ops over N elements
    # fused into one kernel, the gain grows with n and with N
    def chain(n, rows):
        ops = [OpSpec("v0", "exp", ("x",))] + [OpSpec(f"v{i}", "tanh", (f"v{i-1}",)) for i in range(1, n)]
        return GraphSpec("pattern_chain", [TensorSpec("x", "f32", (rows, 256))], ops, [(f"v{n-1}", "f32")])
    f = {(n, rows): B.explore_score(B.Graph.from_spec(chain(n, rows)), list(range(n))) for n in (2, 4) for rows in (64, 8192)}
    assert 0 < f[(2, 64)] < f[(4, 64)] and f[(2, 8192)] < f[(4, 8192)] and f[(2, 64)] < f[(2, 8192)]
    # a tiny tensor: the gain is about the launches (and their memory round trips) saved
    assert f[(4, 64)] > 2.0 * 2.2 and f[(2, 64)] < 2.0 * 3.4
    assert B.explore_score(B.Graph.from_spec(chain(3, 64)), [1]) == 0.0


def test_explorer_errors_and_cycles():
    # A -> B -> C and A -> C: fusing A and C without B would put B between them
    spec = GraphSpec("pattern_tri", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("a", "exp", ("x",)), OpSpec("b", "transpose", ("a",), {"perm": (1, 0)}),
                      OpSpec("bt", "transpose", ("b",), {"perm": (1, 0)}), OpSpec("c", "add", ("a", "bt"))], [("c", "f32")])
    g = B.Graph.from_spec(spec)
    f, f_opt, code = B.explore_score_ex(g, [0, 3])
    assert code == -4 and f is None                     # FS_ERR_CYCLE
    f, f_opt, code = B.explore_score_ex(g, [0, 1])
    assert code == -5 and f_opt > 0                     # convex, but no kernel runs exp + transpose
    prog = B.Program(g)
    assert sorted(len(p["ops"]) for p in prog.patterns()) == [1, 1, 1, 1]
    with pytest.raises(B.FsError):
        B.explore_score(g, [0, 0])
    with pytest.raises(B.FsError):
        B.explore_score(g, [7])
    # an output stored narrower than computed that also feeds another pattern: refused, with advice
    spec = GraphSpec("pattern_narrow", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("a", "exp", ("x",)), OpSpec("t", "transpose", ("a",), {"perm": (1, 0)})], [("a", "bf16"), ("t", "f32")])
    with pytest.raises(B.FsError) as e:
        B.Program(B.Graph.from_spec(spec))
    assert e.value.code == -3 and "convert" in e.value.text
    lib = B.load()
    assert lib.fs_explore(None, None, None) == -1
    assert lib.fs_program_query(None, None) == -1
    assert lib.fs_program_execute(None, None, None, None, 0, None) == -1
    lib.fs_program_destroy(None)
