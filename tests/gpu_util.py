"""Shared plumbing of the GPU parity tests: run a workload descriptor through the C ABI
and hand back float64 host arrays for comparison with the oracle."""
from __future__ import annotations

import sys

import numpy as np

from oracle import oracle as O
from paper_2009_10924_amd import binding as B

# Comparison bars (max relative error vs the float64 oracle):
#   float32 outputs 1e-5, 16-bit outputs 1e-2; transposes bit-exact.
# `floor` = 0 means strict |got-ref|/|ref| with 0/0 := 0.  Outputs formed by cancelling
# sums (LayerNorm output, the bias-gradient column sums) are judged against
# max(|ref|, rms(ref)): float32 arithmetic carries an absolute error of about 1e-7 of
# the operands, which no kernel can turn into 1e-5 of an output that happens to be ~0.
TOL = {"f32": 1e-5, "f16": 1e-2, "bf16": 1e-2}


def note(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def run_spec(spec, inputs_np, scheme="auto", repeat=1, **opts):
    """Builds graph + plan, uploads inputs, executes `repeat` times, returns ({name: f64 array}, info)."""
    import torch
    g = B.Graph.from_spec(spec)
    plan = B.Plan(g, scheme, **opts)
    dev_in = [B.to_device(inputs_np[t.name], t.dtype) for t in spec.inputs]
    dev_out = B.alloc_outputs(spec)
    for t in dev_out:
        if t.dtype in (torch.float32, torch.float16, torch.bfloat16):
            t.fill_(float("nan"))
        else:
            t.fill_(-1)
    ws = plan.make_workspace()
    results = []
    for _ in range(repeat):
        plan.execute(dev_in, dev_out, ws)
        torch.cuda.synchronize()
        results.append({name: B.to_host(t, dt).copy() for (name, dt), t in zip(spec.outputs, dev_out)})
    for r in results[1:]:
        for name in r:
            assert np.array_equal(r[name].view(np.uint8), results[0][name].view(np.uint8)), f"{name}: not run-to-run identical"
    out = {name: O.to_f64(results[0][name], dt) for name, dt in spec.outputs}
    raw = results[0]
    return out, raw, plan.info, plan


def check(got, ref, dtype, floor=0.0, what=""):
    err = O.max_rel_err(got, ref, floor)
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU result"
    assert err <= TOL[dtype], f"{what}: max rel err {err:.3e} > {TOL[dtype]:.0e}"
    return err


def run_pack(specs, inputs_list, repeat=1):
    """Plans every spec (scheme AUTO), packs the plans, executes the pack; returns ([{name: f64 array}], pack info)."""
    import torch
    plans = [B.Plan(B.Graph.from_spec(s), "auto") for s in specs]
    pack = B.Pack(plans)
    dev_in, dev_out = [], []
    for spec, inp in zip(specs, inputs_list):
        dev_in.append([B.to_device(inp[t.name], t.dtype) for t in spec.inputs])
        outs = B.alloc_outputs(spec)
        for t in outs:
            t.fill_(float("nan"))
        dev_out.append(outs)
    stream = torch.cuda.current_stream().cuda_stream
    call = pack.bind([t.data_ptr() for m in dev_in for t in m], [t.data_ptr() for m in dev_out for t in m], stream)
    results = []
    for _ in range(repeat):
        call()
        torch.cuda.synchronize()
        results.append([{name: B.to_host(t, dt).copy() for (name, dt), t in zip(spec.outputs, outs)}
                        for spec, outs in zip(specs, dev_out)])
    for r in results[1:]:
        for a, b in zip(r, results[0]):
            for name in a:
                assert np.array_equal(a[name].view(np.uint8), b[name].view(np.uint8)), f"{name}: not run-to-run identical"
    out = [{name: O.to_f64(res[name], dt) for name, dt in spec.outputs} for spec, res in zip(specs, results[0])]
    return out, pack.info


def all_candidates(spec, inputs, ref, floors, repeat=1, unfused=True, after_rounding=None):
    """Runs the per-op plan and every stitched candidate of `spec`; returns the worst error per output.
    after_rounding: {output name: 16-bit dtype} for float32 outputs computed from values the graph itself rounded to
    that dtype: near a rounding tie float32 and float64 upstream arithmetic pick different neighbours, so such an output
    is held to the 16-bit bar."""
    after_rounding = after_rounding or {}
    worst = {}
    g = B.Graph.from_spec(spec)
    n = B.Plan(g, "auto").info["n_candidates"]
    runs = ([("unfused", {})] if unfused else []) + [("auto", {"candidate": i}) for i in range(n)]
    for scheme, opts in runs:
        note(f"  case {spec.name} scheme={scheme} opts={opts}")
        try:
            got, _, info, _ = run_spec(spec, inputs, scheme, repeat=repeat, **opts)
        except B.FsError as e:
            # a generated kernel whose launch shape holds more per lane than the register file: the library
            # refuses the shape when it is asked for by index (AUTO moves on to the next candidate)
            if "scratch memory" in e.text:
                note(f"  case {spec.name} opts={opts}: refused, {e.text}")
                continue
            raise
        for name, dt in spec.outputs:
            e = check(got[name], ref[name], after_rounding.get(name, dt), floors.get(name, 0.0), f"{spec.name}/{info['kernel']}/{name}")
            worst[name] = max(worst.get(name, 0.0), e)
    return worst
