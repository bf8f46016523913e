"""fs_execute_static (the entry point for callers that cannot allocate): same results as fs_execute.

Two calls in a row on one GPU, the second with a smaller input, so the static scratch array still holds the first
call's partial sums when the second runs; a different pattern (LayerNorm backward, other scratch layout) follows.
Every output is compared bit for bit with fs_execute on a caller-owned workspace, and with the float64 oracle at
the usual bars (float32 1e-5 over max(|ref|, rms) for the column sums, 16-bit outputs 1e-2).
"""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2009_10924_amd import binding as B
from workloads import bias_gelu_dbias_graph, layernorm_backward_graph, make_inputs

from tests.gpu_util import TOL, note

pytestmark = pytest.mark.gpu

CANCELLING = {"dbias", "dgamma", "dbeta", "dx"}   # outputs formed by signed sums: judged over max(|ref|, rms(ref))


def _both_ways(spec, seed):
    import torch
    inp = make_inputs(spec, seed=seed)
    plan = B.Plan(B.Graph.from_spec(spec), "auto")
    assert 0 < plan.info["workspace_bytes"] <= B.FS_STATIC_SCRATCH_BYTES, plan.info
    dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
    stream = torch.cuda.current_stream().cuda_stream
    results = []
    for static in (False, True):
        outs = B.alloc_outputs(spec)
        for t in outs:
            t.fill_(float("nan"))
        if static:
            plan.execute_static_ptrs([t.data_ptr() for t in dev_in], [t.data_ptr() for t in outs], stream)
        else:
            plan.execute(dev_in, outs, plan.make_workspace())
        torch.cuda.synchronize()
        results.append({name: B.to_host(t, dt).copy() for (name, dt), t in zip(spec.outputs, outs)})
    ref = O.evaluate(spec, inp)
    for name, dt in spec.outputs:
        a, b = results[0][name], results[1][name]
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), f"{spec.name}/{name}: static scratch differs from the workspace call"
        got = O.to_f64(b, dt)
        floor = O.rms(ref[name]) if name in CANCELLING else 0.0
        err = O.max_rel_err(got, ref[name].reshape(got.shape), floor)
        note(f"  {spec.name}/{name} via fs_execute_static ({plan.info['kernel']}, scratch {plan.info['workspace_bytes']} B): max rel err {err:.3e}")
        assert np.isfinite(got).all() and err <= TOL[dt], (spec.name, name, err)


def test_static_scratch_two_calls_in_a_row_then_another_pattern():
    note("case fs_execute_static bias_gelu_dbias 2048x3072 bf16")
    _both_ways(bias_gelu_dbias_graph(2048, 3072, "bf16"), seed=0)
    note("case fs_execute_static bias_gelu_dbias 300x1032 bf16 (smaller, ragged)")
    _both_ways(bias_gelu_dbias_graph(300, 1032, "bf16"), seed=1)
    note("case fs_execute_static layernorm_backward 1024x768 f32")
    _both_ways(layernorm_backward_graph(1024, 768, "f32"), seed=2)


def test_static_scratch_refuses_what_does_not_fit():
    import torch
    spec = bias_gelu_dbias_graph(4096, 3072, "bf16")
    plan = B.Plan(B.Graph.from_spec(spec), "unfused")    # float32 intermediates of the per-op plan: far beyond the array
    assert plan.info["workspace_bytes"] > B.FS_STATIC_SCRATCH_BYTES
    inp = make_inputs(spec, seed=0)
    dev_in = [B.to_device(inp[t.name], t.dtype) for t in spec.inputs]
    outs = B.alloc_outputs(spec)
    with pytest.raises(B.FsError) as e:
        plan.execute_static_ptrs([t.data_ptr() for t in dev_in], [t.data_ptr() for t in outs], torch.cuda.current_stream().cuda_stream)
    assert e.value.code == -7 and "static array holds" in e.value.text
