"""Run as a child process by tests/test_host_sanitizers.py with the sanitizer build of the host core loaded
(FUSION_STITCHING_LIB) and the sanitizer runtime preloaded.  Plans and "executes" the benchmark configurations, the
generic patterns, packs and explored programs through the host stub: every launch is checked and counted, none runs,
no device pointer is dereferenced.  Any AddressSanitizer / UndefinedBehaviorSanitizer report aborts the process."""
import ctypes
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from paper_2009_10924_amd import binding as B                                            # noqa: E402
from workloads import (EXPLORE_CONFIGS, FULL_CONFIGS, GENERIC_CONFIGS, NEXT_CONFIGS, PACK_CONFIGS, gelu_backward_graph,  # noqa: E402
                       independent_tiny_patterns_graph, layernorm_backward_bias_graph, random_multi_pattern, random_row_pattern)


def fake(n, base):
    return [base * (i + 1) for i in range(n)]


def run_plan(spec, scheme="auto", **opts):
    plan = B.Plan(B.Graph.from_spec(spec), scheme, **opts)
    ws = plan.info["workspace_bytes"]
    plan.execute_ptrs(fake(len(spec.inputs), 0x10000), fake(len(spec.outputs), 0x1000000), 0x40000000 if ws else 0, ws, 0)
    if 0 < ws <= B.FS_STATIC_SCRATCH_BYTES:
        plan.execute_static_ptrs(fake(len(spec.inputs), 0x10000), fake(len(spec.outputs), 0x1000000), 0)
    plan.describe()
    plan.source()
    return plan


def run_program(spec, **opts):
    prog = B.Program(B.Graph.from_spec(spec), **opts)
    ws = prog.info["workspace_bytes"]
    ins, outs = fake(len(spec.inputs), 0x10000), fake(len(spec.outputs), 0x1000000)
    prog.bind(ins, outs, 0x40000000, ws, 0)()
    for stage in range(prog.info["n_stages"]):
        prog.bind_stage(stage, ins, outs, 0x40000000, ws, 0)()
    prog.describe()
    prog.patterns()
    return prog


def main():
    lib = B.load()
    lib.fs_stub_launch_count.restype = ctypes.c_long
    assert "host_san" in B.lib_path()
    for compile_ok in ("", "1"):
        if compile_ok:
            os.environ["FS_STUB_COMPILE_OK"] = "1"      # generated kernels "compile": the generator's whole path runs
        for name, make in list(FULL_CONFIGS.items()) + list(NEXT_CONFIGS.items()) + list(GENERIC_CONFIGS.items()):
            spec = make()
            plan = run_plan(spec)
            n = plan.info["n_candidates"]
            for i in range(n):                          # every enumerated launch shape
                try:
                    run_plan(spec, candidate=i)
                except B.FsError as e:
                    assert e.code == -5, (name, i, e)   # a generated candidate that did not "compile"
            run_plan(spec, "unfused")
        for r, c, dt in ((64, 128, "f32"), (37, 96, "bf16"), (300, 1001, "f16")):
            run_plan(gelu_backward_graph(r, c - c % 8 if dt != "f32" else c - c % 4, dt))
            run_plan(layernorm_backward_bias_graph(r, 96, dt, sum_dtype="f32"))
        for seed in range(12):
            run_plan(random_row_pattern(seed, 33, 136, ("f32", "f16", "bf16")[seed % 3], n_ops=6 + seed, column_sums=seed % 3))
        members = PACK_CONFIGS["P1"]()
        pack = B.Pack([B.Plan(B.Graph.from_spec(m), "auto") for m in members])
        pack.bind(fake(sum(len(m.inputs) for m in members), 0x10000), fake(sum(len(m.outputs) for m in members), 0x1000000), 0)()
        for name in ("T1", "T2", "T3"):
            spec = EXPLORE_CONFIGS[name]()
            for opts in ({}, {"no_joint_folds": True}, {"no_packing": True, "no_remote_fusion": True}, {"top_k": 1, "beam_width": 1}):
                run_program(spec, **opts)
        run_program(independent_tiny_patterns_graph())
        for seed in range(6):
            run_program(random_multi_pattern(seed, rows=64, cols=128, segments=2 + seed % 3, column_sums=seed % 2, external_links=seed % 2 == 1))
    # error paths must leave nothing behind either
    g = B.Graph.from_spec(FULL_CONFIGS["C4"]())
    for bad in (lambda: B.Plan(g, "lds"), lambda: B.Plan(g, "auto", candidate=999), lambda: run_plan(FULL_CONFIGS["C4"](), "auto", block_threads=96)):
        try:
            bad()
        except B.FsError:
            pass
    launches = lib.fs_stub_launch_count()
    assert launches > 1000, launches
    print(f"host sanitizer driver: {launches} checked launches, no report")


if __name__ == "__main__":
    main()
