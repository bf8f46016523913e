"""HIP graph capture of the library's launches: fs_execute, fs_pack_execute and fs_program_execute only enqueue
kernels on the caller's stream (no allocation, no synchronisation, no memset), so a caller can capture them into a
graph and replay it.  Every replay is compared with the eager result, with eager work and synchronisations between
the replays."""
import numpy as np
import pytest

from paper_2009_10924_amd import binding as B
from workloads import (FULL_CONFIGS, add_bias_layernorm_graph, bias_gelu_dbias_graph, independent_tiny_patterns_graph,
                       make_inputs, transformer_block_graph)

pytestmark = pytest.mark.gpu


def _capture_and_replay(call, outputs, eager_scramble):
    import torch
    side = torch.cuda.Stream()
    # eager reference
    call(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = [t.clone() for t in outputs]
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(side.cuda_stream)                       # warm the stream outside capture
    side.synchronize()
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream().cuda_stream)
    for k in range(4):
        for t in outputs:
            t.fill_(float("nan"))
        eager_scramble(k)                            # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outputs, want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), f"replay {k} differs from the eager run"


def _buffers(spec, seed=0):
    inp = make_inputs(spec, seed=seed)
    return [B.to_device(inp[t.name], t.dtype) for t in spec.inputs], B.alloc_outputs(spec)


def test_plan_with_two_launches_and_workspace_under_capture():
    import torch
    spec = bias_gelu_dbias_graph(1000, 520)                      # main kernel + fold launch, partials in the workspace
    plan = B.Plan(B.Graph.from_spec(spec), "auto")
    assert plan.info["n_kernels"] == 2
    ins, outs = _buffers(spec)
    ws = plan.make_workspace()
    other = B.Plan(B.Graph.from_spec(add_bias_layernorm_graph(64, 256)), "auto")
    oin, oout = _buffers(add_bias_layernorm_graph(64, 256))

    def call(stream):
        plan.bind([t.data_ptr() for t in ins], [t.data_ptr() for t in outs], ws.data_ptr(), ws.numel(), stream)()

    def scramble(k):
        other.execute(oin, oout, None)
    _capture_and_replay(call, outs, scramble)


def test_packed_launch_and_explored_program_under_capture():
    import torch
    spec = independent_tiny_patterns_graph()
    prog = B.Program(B.Graph.from_spec(spec))
    assert prog.info["n_packs"] == 1
    ins, outs = _buffers(spec)
    ws = prog.make_workspace()

    def call(stream):
        prog.bind([t.data_ptr() for t in ins], [t.data_ptr() for t in outs], ws.data_ptr(), ws.numel(), stream)()
    _capture_and_replay(call, outs, lambda k: ins[0].mul_(1.0))

    spec = transformer_block_graph(3, 40, 4, 32, 256, "bf16")
    prog2 = B.Program(B.Graph.from_spec(spec))
    ins2, outs2 = _buffers(spec)
    ws2 = prog2.make_workspace()

    def call2(stream):
        prog2.bind([t.data_ptr() for t in ins2], [t.data_ptr() for t in outs2], ws2.data_ptr(), ws2.numel(), stream)()
    _capture_and_replay(call2, outs2, lambda k: ins2[0].mul_(1.0))


def test_program_with_joint_fold_launch_under_capture():
    """The backward block: generated kernels with column sums, their partial sums in the plans' workspaces, and the
    one fold launch behind the last step that finishes all of them."""
    if not B.codegen_available():
        pytest.skip("column sums inside patterns need the run-time compiler")
    from workloads import transformer_block_backward_graph
    spec = transformer_block_backward_graph(3, 40, 4, 32, 256, "bf16")
    prog = B.Program(B.Graph.from_spec(spec))
    assert prog.info["n_joint_folds"] >= 2
    ins, outs = _buffers(spec)
    ws = prog.make_workspace()

    def call(stream):
        prog.bind([t.data_ptr() for t in ins], [t.data_ptr() for t in outs], ws.data_ptr(), ws.numel(), stream)()
    _capture_and_replay(call, outs, lambda k: ins[0].mul_(1.0))


def test_row_worked_through_in_chunks_under_capture():
    if not B.codegen_available():
        pytest.skip("rows of this length exist as generated kernels only")
    from workloads import softmax_graph
    spec = softmax_graph(6, 70000, "bf16")
    plan = B.Plan(B.Graph.from_spec(spec), "auto")
    assert "chunks" in plan.info["kernel"]
    ins, outs = _buffers(spec)

    def call(stream):
        plan.bind([t.data_ptr() for t in ins], [t.data_ptr() for t in outs], 0, 0, stream)()
    _capture_and_replay(call, outs, lambda k: ins[0].mul_(1.0))


@pytest.mark.parametrize("generated", [False, True])
def test_row_program_under_capture(generated):
    """The interpreted form (register file beyond 64 KB of LDS) and the generated kernel (launched through its
    module handle; the module was loaded when the plan was made)."""
    from workloads import layernorm_stats_graph
    spec = layernorm_stats_graph(5, 4096, in_dtype="f32", out_dtype="f16", with_variance=True)
    with B.codegen(generated):
        plan = B.Plan(B.Graph.from_spec(spec), "auto")
    assert plan.info["pattern"] == ("row_generated" if generated else "row_program")
    ins, outs = _buffers(spec)

    def call(stream):
        plan.bind([t.data_ptr() for t in ins], [t.data_ptr() for t in outs], 0, 0, stream)()
    _capture_and_replay(call, outs, lambda k: ins[0].mul_(1.0))
