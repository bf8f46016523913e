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
# Below the smallest normal number of the storage dtype the spacing of representable values is absolute, not
# relative (float16: 2^-24 under 2^-14), so a result there is judged against that smallest normal number: the
# 1e-2 bar of a float16 output then allows 6e-7 of absolute error, ten float16 subnormal steps.
MIN_NORMAL = {"f32": 2.0 ** -126, "f16": 2.0 ** -14, "bf16": 2.0 ** -126}

_NONNEG_OPS = {"exp", "square", "abs", "sigmoid", "relu", "sqrt", "rsqrt"}
_PASS_THROUGH = {"broadcast", "transpose"}


def cancelling_outputs(spec, inputs):
    """Names of the outputs whose value may be a difference of nearly equal computed terms, derived from the
    descriptor: these, and only these, are judged against max(|ref|, rms(ref)) instead of |ref|.

    float32 arithmetic gives every computed value a relative error of about 1e-7.  An `add` / `sub` / `add_scalar`
    whose result can be near zero while an operand is a computed (already rounded) value, a `reduce_sum` /
    `reduce_mean` over values of both signs, and a `log` (whose result is near zero for arguments near one) turn
    that into an error that is small against the operands but unbounded against the result (the derivative of the
    tanh-GELU likewise: it changes sign near -0.752, where its two terms cancel); every op that passes
    relative error on (mul, div, scale, max, square, abs, relu, sqrt, rsqrt, tanh, the GELU pair, reduce_max,
    convert, broadcast, transpose) passes the property on.  `exp` and `sigmoid` end it (their relative error is the
    absolute error of the argument), and so do sums of non-negative terms.  Sums of graph inputs are exact to half
    an ulp of the result and do not cancel in this sense.  Signs of graph inputs are read from the data."""
    exact, nonneg, cancel = {}, {}, {}
    for t in spec.inputs:
        a = O.to_f64(inputs[t.name], t.dtype)
        exact[t.name], nonneg[t.name], cancel[t.name] = True, bool((a >= 0).all()), False
    for op in spec.ops:
        e = [exact[n] for n in op.inputs]
        nn = [nonneg[n] for n in op.inputs]
        c = [cancel[n] for n in op.inputs]
        code = op.opcode
        if code in ("add", "sub"):
            sum_of_nonneg = code == "add" and all(nn)
            out = (False, sum_of_nonneg, (any(c) or not all(e)) and not sum_of_nonneg)
        elif code == "add_scalar":
            keeps_sign = nn[0] and op.attr["value"] >= 0
            out = (False, keeps_sign, (c[0] or not e[0]) and not keeps_sign)
        elif code == "scale":
            out = (False, nn[0] and op.attr["value"] >= 0, c[0])
        elif code in ("mul", "div"):
            out = (False, all(nn), any(c))
        elif code == "max":
            out = (all(e), any(nn), any(c))
        elif code in ("exp", "sigmoid"):
            out = (False, True, False)
        elif code in _NONNEG_OPS:
            out = (False, True, c[0])
        elif code in ("tanh", "gelu_tanh"):
            out = (False, False, c[0])      # zero only at zero, where they behave like their argument
        elif code in ("log", "gelu_tanh_grad"):
            out = (False, False, True)      # zero at a generic argument (1; about -0.752): a sum of terms that cancel there
        elif code in ("reduce_sum", "reduce_mean"):
            out = (False, nn[0], not nn[0])
        elif code == "reduce_max":
            out = (e[0], nn[0], c[0])
        elif code in _PASS_THROUGH:
            out = (e[0], nn[0], c[0])
        elif code == "convert":
            out = (False, nn[0], c[0])
        else:
            raise ValueError(f"cancelling_outputs: unknown opcode {code}")
        exact[op.out], nonneg[op.out], cancel[op.out] = out
    return {name for name, _ in spec.outputs if cancel[name]}


def floors_for(spec, inputs, ref):
    """{output name: rms(ref)} for the outputs that cancelling_outputs names; the others are strict."""
    names = cancelling_outputs(spec, inputs)
    return {name: O.rms(ref[name]) for name in names}


def stored_converts(spec):
    """Names of `convert` results that are graph outputs and are read by other ops of the graph."""
    outs = {name for name, _ in spec.outputs}
    return [op.out for op in spec.ops if op.opcode == "convert" and op.out in outs and any(op.out in o.inputs for o in spec.ops)]


def reference_given_stored(spec, inputs, raw):
    """The oracle's outputs with every stored_converts() tensor downstream replaced by what the GPU stored for it
    (raw: {output name: storage array}): an output computed from a value that the graph itself rounded to 16 bits
    is then held to its own bar, whichever neighbour a rounding tie upstream went to."""
    dts = dict(spec.outputs)
    names = stored_converts(spec)
    return O.evaluate(spec, inputs, stored={n: O.to_f64(raw[n], dts[n]) for n in names}) if names else O.evaluate(spec, inputs)


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
    err = O.max_rel_err(got, ref, max(floor, MIN_NORMAL[dtype]))
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


def all_candidates(spec, inputs, ref, floors, repeat=1, unfused=True):
    """Runs the per-op plan and every stitched candidate of `spec`; returns the worst error per output.
    Outputs computed from a `convert` result that is itself a graph output are compared with the oracle evaluated on
    the values this run stored for that result (reference_given_stored); the stored result itself with the plain
    oracle."""
    worst = {}
    g = B.Graph.from_spec(spec)
    n = B.Plan(g, "auto").info["n_candidates"]
    runs = ([("unfused", {})] if unfused else []) + [("auto", {"candidate": i}) for i in range(n)]
    resample = bool(stored_converts(spec))
    for scheme, opts in runs:
        note(f"  case {spec.name} scheme={scheme} opts={opts}")
        try:
            got, raw, info, _ = run_spec(spec, inputs, scheme, repeat=repeat, **opts)
        except B.FsError as e:
            # a generated kernel whose launch shape holds more per lane than the register file: the library
            # refuses the shape when it is asked for by index (AUTO moves on to the next candidate)
            if "scratch memory" in e.text:
                note(f"  case {spec.name} opts={opts}: refused, {e.text}")
                continue
            raise
        ref_run = reference_given_stored(spec, inputs, raw) if resample else ref
        for name, dt in spec.outputs:
            e = check(got[name], ref_run[name].reshape(got[name].shape), dt, floors.get(name, 0.0), f"{spec.name}/{info['kernel']}/{name}")
            worst[name] = max(worst.get(name, 0.0), e)
    return worst
