"""Host side of the code generator (Section 4: a fusion pattern becomes one kernel): the generated HIP source,
its compilation by the run-time compiler (needs no GPU), the process-wide switch and the listing calls."""
import re

import pytest

from paper_2009_10924_amd import binding as B
from workloads import (layernorm_stats_graph, masked_scores_gate_graph, random_multi_pattern, random_row_pattern,
                       silu_gate_graph, softmax_graph)
from workloads.graphs import GraphSpec, OpSpec, TensorSpec

pytestmark = pytest.mark.skipif(not B.codegen_available(), reason="the HIP run-time compiler is not installed here")


def _plan(spec, **opts):
    return B.Plan(B.Graph.from_spec(spec), "auto", **opts)


def test_switch_controls_which_candidates_are_offered():
    spec = layernorm_stats_graph(64, 768, with_variance=True)
    before = B.codegen_enable(True)
    try:
        with B.codegen(True):
            on = _plan(spec)
        with B.codegen(False):
            off = _plan(spec)
            assert B.codegen_enable(False) is False          # reports the setting it replaces
        kinds_on = [c["pattern"] for c in on.candidates()]
        kinds_off = [c["pattern"] for c in off.candidates()]
        assert set(kinds_off) == {"row_program"}
        # interpreted candidates first and unchanged, generated ones after them
        assert kinds_on[:len(kinds_off)] == kinds_off and set(kinds_on[len(kinds_off):]) == {"row_generated"}
        assert on.info["pattern"] == "row_generated" and off.info["pattern"] == "row_program"
        assert off.source() == ""
    finally:
        B.codegen_enable(before)


def test_generated_source_is_specialised_to_pattern_extents_and_shape():
    spec = layernorm_stats_graph(100, 768, in_dtype="f32", out_dtype="bf16", with_variance=True)
    plan = _plan(spec)
    info, src = plan.info, plan.source()
    assert info["pattern"] == "row_generated" and info["n_kernels"] == 1 and info["workspace_bytes"] == 0
    m = re.search(r"typedef GenRow<(\d+)u, (\d+)u, (\d+), (\d+), (\d+)u, (true|false), 1u, 768u> Row;", src)
    assert m, src
    rows, cols, vec, k, lanes, block = int(m[1]), int(m[2]), int(m[3]), int(m[4]), int(m[5]), m[6] == "true"
    assert (rows, cols, vec) == (100, 768, 4)
    assert k == info["vecs_per_lane"] and (256 if block else lanes) == info["lanes_per_row"]
    assert lanes * k * vec >= cols                           # the row fits its lanes
    # one load per input, every load before the first arithmetic, one store per output
    body = src.splitlines()
    first_math = min(i for i, l in enumerate(body) if "acc[j] = acc[j]" in l)
    loads = [i for i, l in enumerate(body) if "row.load<" in l]
    assert len(loads) == 5 and max(loads) < first_math
    assert src.count("row.store<bf16_t>") == 1 and src.count("row.store_scalar<float>") == 3
    assert src.count("row.reduce<OpSum") == 2 and "true>(acc" in src      # the variance reduction squares on the fly
    # the compiled kernel's own register count, read from the code object: no GPU needed
    assert 16 <= info["vgprs"] <= 256


def test_every_generated_candidate_compiles_and_reports_registers():
    spec = silu_gate_graph(64, 4096, "bf16")
    n = _plan(spec).info["n_candidates"]
    seen = 0
    for i in range(n):
        try:
            p = _plan(spec, candidate=i)
        except B.FsError as e:
            assert "scratch memory" in e.text                # a shape that would spill is refused by index
            continue
        if p.info["pattern"] == "row_generated":
            seen += 1
            assert p.info["vgprs"] > 0 and "fs_gen_row_" in p.source()
    assert seen >= 2


def _force_every_generated_candidate(spec):
    """AUTO falls back to another candidate when a generated kernel does not compile; asking for the candidate by
    index turns such a failure into an error, so a mistake in the generator cannot hide behind the fallback."""
    g = B.Graph.from_spec(spec)
    n = B.Plan(g, "auto").info["n_candidates"]
    seen = 0
    for i in range(n):
        try:
            p = B.Plan(g, "auto", candidate=i)
        except B.FsError as e:
            assert "scratch memory" in e.text, f"{spec.name} candidate {i}: {e.text[:2000]}"
            continue
        seen += p.info["pattern"] == "row_generated"
    return seen


def test_generated_source_compiles_for_every_kind_of_operand():
    from workloads import (bias_head_split_graph, gelu_backward_graph, head_merge_residual_graph, normalize_from_stats_graph, outer_scale_graph,
                           rmsnorm_backward_graph,
                           scaled_softmax_colbias_graph, transpose_chain_stats_graph, transposed_softmax_graph)
    specs = [layernorm_stats_graph(24, 96, in_dtype="bf16", out_dtype="f16", with_variance=True),
             silu_gate_graph(9, 64, "f16"), scaled_softmax_colbias_graph(13, 40, "f32"),
             normalize_from_stats_graph(11, 48, "bf16"), outer_scale_graph(7, 16),
             masked_scores_gate_graph(2, 3, 5, 64, dtype="bf16"),
             bias_head_split_graph(2, 5, 3, 16, "bf16"), head_merge_residual_graph(2, 5, 3, 64, "f16"),   # column vector + permuted rows
             transpose_chain_stats_graph(2, 5, 3, 16), transposed_softmax_graph(2, 5, 3, 32, "f16"),
             layernorm_stats_graph(3, 4096, in_dtype="f32", out_dtype="f32", with_variance=True),           # workgroup per row
             gelu_backward_graph(300, 96, "bf16"), rmsnorm_backward_graph(5000, 2048, "f16")]               # column sums, both row forms
    for spec in specs:
        assert _force_every_generated_candidate(spec) >= 1, spec.name


def test_stretched_operands_and_scalars_appear_as_constants():
    spec = masked_scores_gate_graph(2, 3, 16, 64, dtype="f16")
    src = _plan(spec).source()
    assert "row.row_c / 16u" in src and "/ 3u" in src and "lead0 * 1u" in src      # the row's index along the leading axes, by constant divisors
    assert "row.load<f16_t, false>(a.full[1]" in src         # the mask is re-read by many rows: cached load
    assert "row.load<f16_t, true>(a.full[0]" in src          # the scores stream
    assert re.search(r"0x41f00000u /\* 30 \*/", src)         # the immediate, bit-exact


def test_kernel_names_tell_patterns_and_shapes_apart():
    """The entry point's name carries a hash of the source: two shapes of one pattern, or two patterns, get two
    names (kernel traces list them separately); the same plan made twice gets the same name."""
    spec = layernorm_stats_graph(64, 768, with_variance=True)

    def entry(plan):
        return [l.split()[1] for l in plan.describe().splitlines() if l.strip().startswith("entry ")][0]

    a, b = _plan(spec), _plan(spec)
    assert entry(a) == entry(b) and entry(a).startswith("fs_gen_row_") and entry(a) in a.source()
    gen = [c["candidate"] for c in a.candidates() if c["pattern"] == "row_generated"]
    names = {entry(_plan(spec, candidate=i)) for i in gen}
    assert len(names) == len(gen)
    assert entry(_plan(silu_gate_graph(64, 768, "f32"))) not in names


def test_patterns_of_hand_written_families_keep_their_kernels():
    info = _plan(softmax_graph(64, 128, "f32")).info
    assert info["pattern"] == "softmax" and not info["kernel"].startswith("row_generated")


@pytest.mark.parametrize("seed", [3, 17, 42])
def test_random_patterns_generate_and_compile(seed):
    spec = random_row_pattern(seed, 37, 96, "f32", n_ops=6 + seed % 12)     # ragged: 37 rows, 24 vectors per row
    plan = _plan(spec)
    assert plan.info["pattern"] == "row_generated", plan.info
    assert plan.source().count("row.store") == len(spec.outputs)


def test_explorer_compiles_only_what_the_chosen_plan_runs():
    spec = random_multi_pattern(5, 24, 64, segments=3, dtype="f32", seg_ops=(4, 8))
    g = B.Graph.from_spec(spec)
    with B.codegen(True):
        prog = B.Program(g)
    kinds = [p["info"]["pattern"] for p in prog.patterns()]
    assert "row_generated" in kinds
    with B.codegen(False):
        prog_off = B.Program(g)
    assert "row_generated" not in [p["info"]["pattern"] for p in prog_off.patterns()]
    assert prog.info["n_ops"] == prog_off.info["n_ops"]


def test_unsupported_pattern_is_not_rescued_by_code_generation():
    # a column sum that the pattern itself reads again would take a grid-wide wait inside the kernel
    spec = GraphSpec("pattern_x", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("s", "reduce_sum", ("e",), {"axis": 0}), OpSpec("y", "div", ("e", "s"))],
                     [("y", "f32")])
    assert _plan(spec).info["scheme"] == "unfused"
    # as an output it is fine: partial sums + fold
    spec = GraphSpec("pattern_x", [TensorSpec("x", "f32", (8, 16))],
                     [OpSpec("e", "exp", ("x",)), OpSpec("s", "reduce_sum", ("e",), {"axis": 0})], [("s", "f32")])
    assert _plan(spec).info["scheme"] == "global"


def test_fall_back_when_compilation_fails(monkeypatch):
    """With every compilation reported as failed: AUTO moves to the interpreted candidate; a pattern whose only
    stitched form is a generated kernel runs per op (plan and explored program alike); by index the failure is an
    error; a pack falls back to the fixed packed kernel."""
    from workloads import gelu_backward_graph
    monkeypatch.setenv("FS_CODEGEN_INJECT_FAILURE", "1")
    spec = layernorm_stats_graph(64, 768, with_variance=True)
    plan = _plan(spec)
    assert plan.info["pattern"] == "row_program" and plan.source() == ""
    generated = [c["candidate"] for c in plan.candidates() if c["pattern"] == "row_generated"]
    with pytest.raises(B.FsError) as e:
        _plan(spec, candidate=generated[0])
    assert e.value.code == -5 and "injected" in e.value.text
    colsum = gelu_backward_graph(300, 96, "bf16")          # no interpreted form
    info = _plan(colsum).info
    assert info["scheme"] == "unfused" and info["n_kernels"] >= len(colsum.ops)    # (the column sum takes two launches)
    prog = B.Program(B.Graph.from_spec(colsum))
    assert prog.info["n_kernels"] >= 2 and "row_generated" not in [p["info"]["pattern"] for p in prog.patterns()]
    pack = B.Pack([_plan(softmax_graph(64, 128, "f32")), _plan(softmax_graph(9, 256, "f32"))])
    assert pack.info["generated"] == 0 and pack.info["n_kernels"] == 1
    monkeypatch.delenv("FS_CODEGEN_INJECT_FAILURE")
    assert _plan(spec).info["pattern"] == "row_generated"


def test_code_objects_survive_the_process_in_the_cache_directory(tmp_path):
    """FS_CODEGEN_CACHE_DIR: the first process compiles and leaves a file, the second one loads it (and says the same
    about the kernel); a damaged file is a miss, not an error."""
    import os
    import subprocess
    import sys
    script = ("import time; t0 = time.time();"
              "from paper_2009_10924_amd import binding as B; from workloads import layernorm_stats_graph;"
              "p = B.Plan(B.Graph.from_spec(layernorm_stats_graph(64, 768, with_variance=True)));"
              "print(p.info['pattern'], p.info['vgprs'])")
    env = dict(os.environ, FS_CODEGEN_CACHE_DIR=str(tmp_path))
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    first = subprocess.run([sys.executable, "-c", script], cwd=root, env=env, capture_output=True, text=True, check=True).stdout.split()
    files = sorted(tmp_path.glob("fs_gfx950_*.co"))
    assert first[0] == "row_generated" and len(files) == 1 and files[0].stat().st_size > 4096
    stamp = files[0].stat().st_mtime_ns
    second = subprocess.run([sys.executable, "-c", script], cwd=root, env=env, capture_output=True, text=True, check=True).stdout.split()
    assert second == first and files[0].stat().st_mtime_ns == stamp          # read, not rewritten
    data = files[0].read_bytes()
    files[0].write_bytes(data[:100] + bytes(50) + data[150:])               # the stored source no longer matches
    third = subprocess.run([sys.executable, "-c", script], cwd=root, env=env, capture_output=True, text=True, check=True).stdout.split()
    assert third == first and files[0].read_bytes() == data                  # compiled again and written back


def test_plans_can_be_made_from_several_threads_at_once():
    """Compilation and the process-wide kernel cache are serialised inside the library: eight threads making plans of
    overlapping patterns all get working plans, and identical sources end up as one kernel (one name)."""
    from concurrent.futures import ThreadPoolExecutor
    specs = [layernorm_stats_graph(32 + 8 * (i % 3), 768, with_variance=True) for i in range(12)] + \
            [silu_gate_graph(16, 256 + 64 * (i % 2), "f32") for i in range(4)]

    def make(spec):
        p = _plan(spec)
        entry = [l.split()[1] for l in p.describe().splitlines() if l.strip().startswith("entry ")]
        return spec.name, p.info["pattern"], entry[0] if entry else ""

    with ThreadPoolExecutor(max_workers=8) as pool:
        results = list(pool.map(make, specs))
    assert all(pattern == "row_generated" and entry for _, pattern, entry in results)
    by_name = {}
    for name, _, entry in results:
        by_name.setdefault(name, set()).add(entry)
    assert all(len(v) == 1 for v in by_name.values())
