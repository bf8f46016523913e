"""Pins for the float64 oracle: closed forms, invariants, brute force, hand-worked fixtures.

Each pin is chosen so that a plausible slip in the oracle (dropped term, wrong
sign, wrong axis, transposed operand, wrong constant) fails at least one test.
None of them calls the oracle to make its own expected value.
"""
import math
import os
import statistics

import numpy as np
import pytest

from oracle import oracle as O
from workloads import (add_bias_layernorm_graph, attention_scores_graph, bias_gelu_dbias_graph,
                       layernorm_backward_graph, make_inputs, quantise, rmsnorm_graph, softmax_backward_graph, softmax_graph,
                       transpose_chain_graph, transpose_graph, valid_lengths)


def _read_rows(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line)
    return rows


# ------------------------------------------------------------------ dtype helpers
def test_bf16_widening_and_rounding_exact():
    # 1.0 = 0x3F80, -2.5 = 0xC020, smallest step above 1 is 2^-7
    bits = np.array([0x3F80, 0xC020, 0x3F81, 0x0000], dtype=np.uint16)
    np.testing.assert_array_equal(O.to_f64(bits, "bf16"), [1.0, -2.5, 1.0 + 2.0 ** -7, 0.0])
    # ties go to the even neighbour: 1 + 2^-8 is halfway between 1 and 1+2^-7 -> 1 ;
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd) and 1+2^-6 (even) -> 1+2^-6
    v = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20, -3.0, 0.0, 1e-3])
    r = O.round_to(v, "bf16")
    assert r[0] == 1.0 and r[1] == 1 + 2.0 ** -6 and r[2] == 1 + 2.0 ** -7 and r[3] == -3.0 and r[4] == 0.0
    # generator's quantiser (integer bit trick) and the oracle's (frexp/rint) agree on random data
    rng = np.random.default_rng(5)
    a = rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))
    np.testing.assert_array_equal(O.to_f64(quantise(a.astype(np.float32).astype(np.float64), "bf16"), "bf16"),
                                  O.round_to(a.astype(np.float32).astype(np.float64), "bf16"))
    # every rounded value is within half a bf16 ulp (2^-8 relative at worst)
    assert np.max(np.abs(O.round_to(a, "bf16") - a) / np.abs(a)) <= 2.0 ** -8


def test_f16_roundtrip():
    a = np.array([1.0, 1.0 + 2.0 ** -11, -10000.0, 65504.0])
    np.testing.assert_array_equal(O.round_to(a, "f16"), [1.0, 1.0, -10000.0, 65504.0])


# ------------------------------------------------------------------ softmax (C1)
def test_softmax_golden_log_rows(golden_dir):
    for line in _read_rows(os.path.join(golden_dir, "softmax_log_rows.txt")):
        a = [float(t) for t in line.split()]
        g = softmax_graph(1, len(a), "f32")
        x = np.log(np.array([a], dtype=np.float64))
        # feed float64 directly (bypass storage rounding): evaluate on a float64 'input'
        y = _eval_f64(g, {"x": x})["y"][0]
        np.testing.assert_allclose(y, np.array(a) / sum(a), rtol=1e-14)


def _eval_f64(graph, f64_inputs):
    """Evaluate with float64 inputs given directly (monkeypatch-free: wrap to_f64)."""
    class _G:
        pass
    g = _G()
    g.inputs = [type(t)(t.name, "f64raw", t.dims) for t in graph.inputs]
    g.ops, g.outputs = graph.ops, graph.outputs
    orig = O.to_f64
    try:
        O.to_f64 = lambda a, dt: np.asarray(a, dtype=np.float64) if dt == "f64raw" else orig(a, dt)
        return O.evaluate(g, f64_inputs)
    finally:
        O.to_f64 = orig


def test_softmax_invariants():
    g = softmax_graph(64, 128, "f32")
    inp = make_inputs(g, seed=0)
    y = O.evaluate(g, inp)["y"]
    assert y.shape == (64, 128)
    np.testing.assert_allclose(y.sum(axis=1), 1.0, atol=1e-12)            # rows sum to 1
    assert (y > 0).all() and (y <= 1).all()
    # shift invariance per row (float64 inputs fed directly, so the shift is not re-rounded)
    x = O.to_f64(inp["x"], "f32")
    shift = np.linspace(-3, 3, 64)[:, None]
    y2 = _eval_f64(g, {"x": x + shift})["y"]
    np.testing.assert_allclose(y2, y, rtol=1e-12)
    # argmax of each row carries the largest probability, ordering preserved
    assert (np.argmax(y, axis=1) == np.argmax(inp["x"], axis=1)).all()
    # ratio property: y_i / y_j = exp(x_i - x_j)
    np.testing.assert_allclose(y[:, 3] / y[:, 17], np.exp(x[:, 3] - x[:, 17]), rtol=1e-12)


def test_softmax_uniform_and_two_element_closed_form():
    g = softmax_graph(2, 8, "f32")
    y = O.evaluate(g, {"x": np.full((2, 8), 3.25, np.float32)})["y"]
    assert (y == 0.125).all()
    g2 = softmax_graph(1, 2, "f32")
    for a, b in [(0.5, -1.25), (2.0, 2.0), (-3.0, 4.0)]:
        y = O.evaluate(g2, {"x": np.array([[a, b]], np.float32)})["y"][0]
        assert y[0] == pytest.approx(1.0 / (1.0 + math.exp(b - a)), rel=1e-14)
        assert y[1] == pytest.approx(1.0 / (1.0 + math.exp(a - b)), rel=1e-14)


def test_softmax_bruteforce_python_loops():
    g = softmax_graph(3, 4, "f32")
    x = np.array([[0.5, -1.0, 2.0, 0.0], [1.0, 1.0, 1.0, -7.5], [-2.0, 3.0, 0.25, 0.75]], np.float32)
    y = O.evaluate(g, {"x": x})["y"]
    for i in range(3):
        row = [float(v) for v in x[i]]
        den = math.fsum(math.exp(v) for v in row)
        for j in range(4):
            assert y[i, j] == pytest.approx(math.exp(row[j]) / den, rel=1e-13)


# ------------------------------------------------------------------ attention scores (C3)
def test_attention_scores_mask_semantics():
    B, H, S, T = 4, 3, 5, 32
    g = attention_scores_graph(B, H, S, T)
    inp = make_inputs(g, seed=0)
    lens = valid_lengths(B, T, seed=0)
    assert ((lens >= 16) & (lens <= T)).all()
    mask = O.to_f64(inp["mask"], "f16")
    assert set(np.unique(mask)) <= {0.0, -10000.0}
    y = O.evaluate(g, inp)["y"]
    s = O.to_f64(inp["scores"], "f16")
    for b in range(B):
        L = int(lens[b])
        assert (mask[b, 0, 0, :L] == 0).all() and (mask[b, 0, 0, L:] == -10000.0).all()
        # masked keys get exactly zero; valid prefix is the plain softmax of the scaled prefix
        assert (y[b, :, :, L:] == 0.0).all()
        for h in range(H):
            for q in range(S):
                row = [0.125 * float(v) for v in s[b, h, q, :L]]
                mx = max(row)
                den = math.fsum(math.exp(v - mx) for v in row)
                want = np.array([math.exp(v - mx) / den for v in row])
                np.testing.assert_allclose(y[b, h, q, :L], want, rtol=1e-13)
    np.testing.assert_allclose(y.sum(axis=-1), 1.0, atol=1e-12)


# ------------------------------------------------------------------ LayerNorm (C2)
def test_layernorm_golden_2x5(golden_dir):
    rows = _read_rows(os.path.join(golden_dir, "layernorm_2x5.txt"))
    data, means, variances = [], [], []
    for line in rows:
        vals, mean, var = [p.strip() for p in line.split("|")]
        data.append([float(t) for t in vals.split()])
        means.append(float(mean))
        variances.append(float(var))
    x = np.array(data, np.float32)
    eps = 1e-5
    g = add_bias_layernorm_graph(2, 5, eps=eps)
    zeros = np.zeros(5, np.float32)
    inp = {"x": x, "res": np.zeros_like(x), "bias": zeros, "gamma": np.ones(5, np.float32), "beta": zeros}
    env = O.evaluate(g, inp, keep_all=True)
    for i in range(2):
        assert env["mu"][i, 0] == pytest.approx(means[i], rel=1e-15)
        assert env["v"][i, 0] == pytest.approx(variances[i], rel=1e-15)
        assert env["v"][i, 0] == pytest.approx(statistics.pvariance(data[i]), rel=1e-15)
        want = [(v - means[i]) / math.sqrt(variances[i] + eps) for v in data[i]]
        np.testing.assert_allclose(env["o"][i], want, rtol=1e-14)


def test_layernorm_invariants_and_affine():
    g = add_bias_layernorm_graph(33, 96)
    inp = make_inputs(g, seed=0)
    env = O.evaluate(g, inp, keep_all=True)
    n, v = env["n"], env["v"]
    np.testing.assert_allclose(n.mean(axis=1), 0.0, atol=1e-12)           # zero mean before the affine step
    np.testing.assert_allclose((n * n).mean(axis=1), (v / (v + 1e-5))[:, 0], rtol=1e-12)  # unit variance up to eps
    # the pre-norm tensor is x + res + bias (all three terms present, bias along columns)
    x, r, b = (O.to_f64(inp[k], "f32") for k in ("x", "res", "bias"))
    np.testing.assert_allclose(env["h"], x + r + b[None, :], rtol=0, atol=1e-15)
    # affine step: o = n * gamma + beta along columns
    ga, be = O.to_f64(inp["gamma"], "f32"), O.to_f64(inp["beta"], "f32")
    np.testing.assert_allclose(env["o"], n * ga[None, :] + be[None, :], rtol=0, atol=1e-15)
    # equivariance: scaling and shifting the row leaves n unchanged up to eps
    inp2 = dict(inp)
    inp2["x"] = (4.0 * O.to_f64(inp["x"], "f32")).astype(np.float32)       # exact in f32
    inp2["res"] = (4.0 * O.to_f64(inp["res"], "f32")).astype(np.float32)
    inp2["bias"] = (4.0 * O.to_f64(inp["bias"], "f32")).astype(np.float32)
    n2 = O.evaluate(g, inp2, keep_all=True)["n"]
    np.testing.assert_allclose(n2, n, rtol=2e-5)       # (v+eps) vs (16v+eps): differs by O(eps/v)
    assert not np.allclose(n2, n, rtol=1e-9)           # ... and eps really is inside the root
    # output reported un-rounded; rounded variant is bf16-exact and within half an ulp
    out = O.evaluate(g, inp)["out"]
    out_r = O.evaluate(g, inp, round_outputs=True)["out"]
    np.testing.assert_array_equal(out, env["o"])
    assert np.max(np.abs(out_r - out) / np.abs(out)) <= 2.0 ** -8
    np.testing.assert_array_equal(O.round_to(out_r, "bf16"), out_r)


# ------------------------------------------------------------------ GELU (C4)
def _gelu(z):
    return O.op_gelu_tanh(np.asarray(z, dtype=np.float64))


def _dgelu(z):
    return O.op_gelu_tanh_grad(np.asarray(z, dtype=np.float64))


def test_gelu_closed_forms_and_identities():
    assert _gelu(0.0) == 0.0 and _dgelu(0.0) == 0.5
    big = np.array([8.0, 12.0, 30.0])
    np.testing.assert_allclose(_gelu(big), big, rtol=1e-15)
    np.testing.assert_allclose(_dgelu(big), 1.0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(_gelu(-big), 0.0, atol=1e-12)
    z = np.linspace(-6, 6, 2401)
    np.testing.assert_allclose(_gelu(z) - _gelu(-z), z, rtol=0, atol=1e-14)       # odd-part identity
    np.testing.assert_allclose(_dgelu(z) + _dgelu(-z), 1.0, rtol=0, atol=1e-14)
    # the tanh form approximates z * Phi(z); its published worst-case gap is a few 1e-4.
    phi = np.array([0.5 * (1.0 + math.erf(v / math.sqrt(2.0))) for v in z])
    gap = np.max(np.abs(_gelu(z) - z * phi))
    assert 1e-4 < gap < 1e-3
    # sigmoid form  z * sigma(2u)  is the same function in exact arithmetic
    u = math.sqrt(2 / math.pi) * (z + 0.044715 * z ** 3)
    sig = 1.0 / (1.0 + np.exp(-2.0 * u))
    inner = np.abs(z) < 3
    np.testing.assert_allclose(_gelu(z)[inner], (z * sig)[inner], rtol=1e-12, atol=1e-300)
    dsig = sig + z * sig * (1 - sig) * 2 * math.sqrt(2 / math.pi) * (1 + 3 * 0.044715 * z * z)
    np.testing.assert_allclose(_dgelu(z)[inner], dsig[inner], rtol=1e-12)


def test_gelu_grad_is_derivative_of_gelu():
    z = np.linspace(-5, 5, 1001)
    h = 1e-6
    fd = (_gelu(z + h) - _gelu(z - h)) / (2 * h)
    np.testing.assert_allclose(_dgelu(z), fd, rtol=0, atol=1e-8)


def _dec_exp(x):
    """exp by its power series in 50-digit decimal arithmetic (argument halved until small, result squared back):
    no library routine for any transcendental is involved."""
    from decimal import Decimal, getcontext
    getcontext().prec = 50
    x = Decimal(x)
    halvings = 0
    while abs(x) > Decimal("0.125"):
        x /= 2
        halvings += 1
    term, total, n = Decimal(1), Decimal(1), 0
    while abs(term) > Decimal(10) ** -48:
        n += 1
        term = term * x / n
        total += term
    for _ in range(halvings):
        total *= total
    return total


def _dec_tanh(x):
    from decimal import Decimal
    e2 = _dec_exp(2 * Decimal(x))
    return (e2 - 1) / (e2 + 1)


def _dec_sqrt_2_over_pi():
    """sqrt(2/pi) with pi from Machin's formula, the arctangents by their series, the root by Newton's iteration."""
    from decimal import Decimal, getcontext
    getcontext().prec = 50

    def arctan_inv(n):
        x = Decimal(1) / n
        term, total, k = x, x, 0
        while abs(term) > Decimal(10) ** -48:
            k += 1
            term = -term * x * x
            total += term / (2 * k + 1)
        return total
    pi = 4 * (4 * arctan_inv(5) - arctan_inv(239))
    r = Decimal(2) / pi
    y = Decimal("0.8")
    for _ in range(8):
        y = (y + r / y) / 2
    return y


def test_series_arithmetic_reproduces_known_constants():
    # the decimal evaluator itself against constants typed from tables (20 digits)
    from decimal import Decimal
    known = {"e": "2.7182818284590452354", "1/e": "0.36787944117144232160", "tanh(1)": "0.76159415595576488812",
             "tanh(1/2)": "0.46211715726000975850", "sqrt(2/pi)": "0.79788456080286535588"}
    got = {"e": _dec_exp(1), "1/e": _dec_exp(-1), "tanh(1)": _dec_tanh(1), "tanh(1/2)": _dec_tanh("0.5"), "sqrt(2/pi)": _dec_sqrt_2_over_pi()}
    for name, text in known.items():
        assert abs(got[name] - Decimal(text)) < Decimal("1e-19"), name


def test_transcendental_ops_against_series_arithmetic():
    """exp, tanh, sigmoid, log, tanh-GELU and its derivative of the oracle against 50-digit series arithmetic that calls
    no library transcendental: a wrong constant (sqrt(2/pi), 0.044715), a dropped term of the derivative or a sign
    error shows at 1e-3 or more; the bar is a few float64 ulps."""
    from decimal import Decimal
    c, k = _dec_sqrt_2_over_pi(), Decimal("0.044715")
    for text in ("-5.5", "-3.5", "-1", "-0.7520", "-0.1", "0", "0.3", "1", "2.5", "6"):
        z = Decimal(text)
        zf = np.array([float(text)])
        u = c * (z + k * z ** 3)
        t = _dec_tanh(u)
        gelu = z * (1 + t) / 2
        grad = (1 + t) / 2 + z * (1 - t * t) / 2 * c * (1 + 3 * k * z * z)
        # (1 + tanh u) cancels in float64 for very negative z (an ulp of tanh near -1, times |z|): an absolute bar
        # of 2e-15 covers that, the relative one everything else
        assert float(O.op_gelu_tanh(zf)[0]) == pytest.approx(float(gelu), rel=2e-14, abs=2e-15)
        assert float(O.op_gelu_tanh_grad(zf)[0]) == pytest.approx(float(grad), rel=2e-14, abs=2e-15)
        assert float(O.op_exp(zf)[0]) == pytest.approx(float(_dec_exp(z)), rel=4e-16)
        assert float(O.op_tanh(zf)[0]) == pytest.approx(float(_dec_tanh(z)), rel=4e-16, abs=1e-300)
        assert float(O.op_sigmoid(zf)[0]) == pytest.approx(float(1 / (1 + _dec_exp(-z))), rel=4e-16)
        # log as the inverse of the series exponential: log(exp(z)) = z
        assert float(O.op_log(np.array([float(_dec_exp(z))]))[0]) == pytest.approx(float(text), rel=4e-16, abs=2e-16)


def test_colsum_golden_7x5(golden_dir):
    rows = _read_rows(os.path.join(golden_dir, "colsum_7x5.txt"))
    mat = np.array([[float(t) for t in r.split()] for r in rows if not r.startswith("sum")])
    want = np.array([float(t) for t in [r for r in rows if r.startswith("sum")][0].split()[1:]])
    got = O.op_reduce_sum(mat, 0)
    assert got.shape == (1, 5)
    np.testing.assert_array_equal(got[0], want)
    # and rows, to catch an axis mix-up
    np.testing.assert_array_equal(O.op_reduce_sum(mat, 1)[:, 0], [math.fsum(r) for r in mat])


def test_bias_gelu_dbias_bruteforce():
    g = bias_gelu_dbias_graph(7, 5)
    inp = make_inputs(g, seed=0)
    out = O.evaluate(g, inp)
    x, b, gr = (O.to_f64(inp[k], "bf16") for k in ("x", "bias", "grad"))
    assert out["y"].shape == (7, 5) and out["dbias"].shape == (1, 5)
    h = 1e-6
    for j in range(5):
        terms = []
        for i in range(7):
            z = float(x[i, j] + b[j])
            assert out["y"][i, j] == pytest.approx(float(_gelu(z)), rel=1e-14)
            fd = (float(_gelu(z + h)) - float(_gelu(z - h))) / (2 * h)
            terms.append(float(gr[i, j]) * fd)
        assert out["dbias"][0, j] == pytest.approx(math.fsum(terms), abs=1e-7)


# ------------------------------------------------------------------ transpose chain (C5)
def test_transpose_involution_and_index_encoding():
    dims, perm = (3, 5, 4, 6), (0, 2, 1, 3)
    g = transpose_graph(dims, perm, "f32")
    inp = make_inputs(g)
    t = O.evaluate(g, inp)["t"]
    assert t.shape == (3, 4, 5, 6)
    # element [b,h,s,d] of the result came from flat index ((b*S+s)*H+h)*D+d of the input
    x = O.to_f64(inp["x"], "f32")
    for b, h, s, d in [(0, 0, 0, 0), (2, 3, 4, 5), (1, 2, 3, 4), (2, 0, 4, 1)]:
        assert t[b, h, s, d] == x.reshape(-1)[((b * 5 + s) * 4 + h) * 6 + d]
    g_back = transpose_graph((3, 4, 5, 6), perm, "f32")
    back = O.evaluate(g_back, {"x": t.astype(np.float32)})["t"]
    np.testing.assert_array_equal(back, x)
    # a perm that moves the last axis
    g2 = transpose_graph((2, 3, 4), (2, 0, 1), "i32")
    t2 = O.evaluate(g2, make_inputs(g2))["t"]
    for i in range(4):
        for j in range(2):
            for k in range(3):
                assert t2[i, j, k] == (j * 3 + k) * 4 + i


def test_transpose_chain_invariants():
    B, S, H, D = 2, 7, 3, 16
    g = transpose_chain_graph(B, S, H, D)
    inp = make_inputs(g, seed=0)
    env = O.evaluate(g, inp, keep_all=True)
    out, ss = env["out"], env["ss"]
    assert out.shape == (B, H, S, D) and ss.shape == (B, H, S, 1)
    np.testing.assert_allclose((out * out).sum(axis=-1, keepdims=True), ss / (ss + 1e-6), rtol=1e-12)
    # brute force one row: out[b,h,s,:] = scale[h] x[b,s,h,:] / sqrt(sum (scale[h] x)^2 + eps)
    x, sc = O.to_f64(inp["x"], "f32"), O.to_f64(inp["scale"], "f32").reshape(-1)
    for b, h, s in [(0, 0, 0), (1, 2, 6), (1, 1, 3)]:
        u = [float(sc[h]) * float(v) for v in x[b, s, h, :]]
        den = math.sqrt(math.fsum(v * v for v in u) + 1e-6)
        np.testing.assert_allclose(out[b, h, s, :], [v / den for v in u], rtol=1e-13)
    # multiplying the scale by k leaves the result unchanged up to eps
    inp2 = dict(inp)
    inp2["scale"] = (2.0 * sc).astype(np.float32).reshape(H, 1, 1)
    out2 = O.evaluate(g, inp2)["out"]
    np.testing.assert_allclose(out2, out, rtol=1e-5)


# ------------------------------------------------------------------ backward patterns
def test_softmax_backward_is_the_gradient_of_softmax():
    rng = np.random.default_rng(11)
    R, C = 3, 6
    x = rng.standard_normal((R, C))
    dy = rng.standard_normal((R, C))
    fwd = softmax_graph(R, C, "f32")
    y = _eval_f64(fwd, {"x": x})["y"]
    bwd = softmax_backward_graph(R, C, "f32")
    dx = _eval_f64(bwd, {"y": y, "dy": dy})["dx"]
    np.testing.assert_allclose(dx.sum(axis=1), 0.0, atol=1e-14)        # rows of dx sum to zero
    h = 1e-6
    for i in range(R):
        for j in range(C):
            xp, xm = x.copy(), x.copy()
            xp[i, j] += h
            xm[i, j] -= h
            lp = float(np.sum(dy * _eval_f64(fwd, {"x": xp})["y"]))
            lm = float(np.sum(dy * _eval_f64(fwd, {"x": xm})["y"]))
            assert dx[i, j] == pytest.approx((lp - lm) / (2 * h), abs=1e-8)
    # a row with a uniform upstream gradient gets exactly zero
    dx0 = _eval_f64(bwd, {"y": y, "dy": np.full((R, C), 2.5)})["dx"]
    np.testing.assert_allclose(dx0, 0.0, atol=1e-15)


def test_layernorm_backward_is_the_gradient_of_layernorm():
    rng = np.random.default_rng(12)
    R, C, eps = 3, 5, 1e-5
    hin = rng.standard_normal((R, C))
    dy = rng.standard_normal((R, C))
    gamma = 1.0 + 0.1 * rng.standard_normal(C)
    fwd = add_bias_layernorm_graph(R, C, eps=eps, out_dtype="f32")
    zeros_rc, zeros_c = np.zeros((R, C)), np.zeros(C)

    def forward(hv, gv):
        return _eval_f64(fwd, {"x": hv, "res": zeros_rc, "bias": zeros_c, "gamma": gv, "beta": zeros_c})["out"]

    mu = hin.mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(((hin - mu) ** 2).mean(axis=1, keepdims=True) + eps)
    bwd = layernorm_backward_graph(R, C, "f32")
    out = _eval_f64(bwd, {"h": hin, "dy": dy, "gamma": gamma, "mu": mu, "rstd": rstd})
    assert out["dx"].shape == (R, C) and out["dgamma"].shape == (1, C) and out["dbeta"].shape == (1, C)
    h = 1e-6
    for i in range(R):
        for j in range(C):
            hp, hm = hin.copy(), hin.copy()
            hp[i, j] += h
            hm[i, j] -= h
            fd = (np.sum(dy * forward(hp, gamma)) - np.sum(dy * forward(hm, gamma))) / (2 * h)
            assert out["dx"][i, j] == pytest.approx(fd, abs=2e-8)
    for j in range(C):
        gp, gm = gamma.copy(), gamma.copy()
        gp[j] += h
        gm[j] -= h
        fd = (np.sum(dy * forward(hin, gp)) - np.sum(dy * forward(hin, gm))) / (2 * h)
        assert out["dgamma"][0, j] == pytest.approx(fd, abs=2e-8)
        assert out["dbeta"][0, j] == pytest.approx(math.fsum(dy[:, j]), abs=1e-14)
    # dx is orthogonal to the constant vector and to x_hat in every row (up to the eps term)
    np.testing.assert_allclose(out["dx"].sum(axis=1), 0.0, atol=1e-13)


def test_rmsnorm_closed_forms():
    eps = 1e-6
    g = rmsnorm_graph(3, 4, eps=eps, dtype="f32")
    x = np.array([[3.0, -4.0, 0.0, 0.0], [1.0, 1.0, 1.0, 1.0], [2.0, -2.0, 2.0, -2.0]])
    gamma = np.array([1.0, 2.0, 0.5, -1.0])
    out = _eval_f64(g, {"x": x, "gamma": gamma})["out"]
    # row 0: mean square = 25/4; row 1: 1; row 2: 4
    for i, ms in enumerate((6.25, 1.0, 4.0)):
        want = [float(x[i, j]) / math.sqrt(ms + eps) * float(gamma[j]) for j in range(4)]
        np.testing.assert_allclose(out[i], want, rtol=1e-14)
    # with gamma = 1 the output has mean square v / (v + eps); scaling x leaves it unchanged up to eps
    ones = np.ones(4)
    o1 = _eval_f64(g, {"x": x, "gamma": ones})["out"]
    np.testing.assert_allclose((o1 ** 2).mean(axis=1), np.array([6.25, 1.0, 4.0]) / (np.array([6.25, 1.0, 4.0]) + eps), rtol=1e-13)
    o2 = _eval_f64(g, {"x": 8.0 * x, "gamma": ones})["out"]
    np.testing.assert_allclose(o2, o1, rtol=1e-6)


# ------------------------------------------------------------------ misc ops + metric
def test_elementwise_ops_against_python_scalars():
    a = np.array([[1.5, -2.0, 0.25], [4.0, 9.0, 16.0]])
    b = np.array([2.0, -0.5, 4.0])
    np.testing.assert_array_equal(O.op_sub(a, b), [[-0.5, -1.5, -3.75], [2.0, 9.5, 12.0]])
    np.testing.assert_array_equal(O.op_div(a, b), [[0.75, 4.0, 0.0625], [2.0, -18.0, 4.0]])
    np.testing.assert_array_equal(O.op_max(a, b), [[2.0, -0.5, 4.0], [4.0, 9.0, 16.0]])
    np.testing.assert_array_equal(O.op_rsqrt(a[1]), [0.5, 1.0 / 3.0, 0.25])
    np.testing.assert_array_equal(O.op_scale(a[0], 2.0), [3.0, -4.0, 0.5])
    np.testing.assert_array_equal(O.op_add_scalar(a[0], 1.0), [2.5, -1.0, 1.25])
    np.testing.assert_array_equal(O.op_square(a[0]), [2.25, 4.0, 0.0625])
    np.testing.assert_array_equal(O.op_reduce_max(a, 1)[:, 0], [1.5, 16.0])
    np.testing.assert_array_equal(O.op_reduce_mean(a, 0)[0], [2.75, 3.5, 8.125])
    assert O.op_exp(np.array([1.0]))[0] == pytest.approx(2.718281828459045, rel=1e-15)      # e and tanh(1/2) typed from tables
    assert O.op_tanh(np.array([0.5]))[0] == pytest.approx(0.46211715726000976, rel=1e-15)
    np.testing.assert_array_equal(O.op_broadcast(b.reshape(1, 3), (2, 3)), [b, b])


def test_log_sigmoid_relu_abs_sqrt_closed_forms():
    x = np.linspace(-6.0, 6.0, 49)
    pos = np.array([1e-6, 0.25, 1.0, 2.0, 9.0, 1e6])
    # python scalars, one by one
    for v in pos:
        assert O.op_log(np.array([v]))[0] == pytest.approx(math.log(v), rel=1e-15, abs=1e-300)
        assert O.op_sqrt(np.array([v]))[0] == pytest.approx(math.sqrt(v), rel=1e-15)
    np.testing.assert_array_equal(O.op_sqrt(np.array([0.0, 4.0, 6.25])), [0.0, 2.0, 2.5])
    np.testing.assert_array_equal(O.op_log(np.array([1.0])), [0.0])
    # identities that a wrong sign, a missing term or a swapped definition breaks
    np.testing.assert_allclose(O.op_log(O.op_exp(x)), x, rtol=0, atol=1e-14)
    np.testing.assert_allclose(O.op_sigmoid(x) + O.op_sigmoid(-x), 1.0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(O.op_sigmoid(x), 0.5 * (1.0 + np.tanh(0.5 * x)), rtol=1e-14)
    assert O.op_sigmoid(np.array([0.0]))[0] == 0.5 and O.op_sigmoid(np.array([math.log(3.0)]))[0] == pytest.approx(0.75, rel=1e-15)
    np.testing.assert_array_equal(O.op_relu(x) - O.op_relu(-x), x)
    np.testing.assert_array_equal(O.op_relu(x) + O.op_relu(-x), O.op_abs(x))
    np.testing.assert_array_equal(O.op_abs(np.array([-1.5, 0.0, 2.0])), [1.5, 0.0, 2.0])
    np.testing.assert_allclose(O.op_sqrt(pos) ** 2, pos, rtol=1e-15)


def test_log_softmax_is_the_logarithm_of_softmax():
    from workloads import log_softmax_graph, softmax_graph
    rng = np.random.default_rng(5)
    x = rng.normal(0.0, 3.0, (7, 33))
    ls = O.evaluate(log_softmax_graph(7, 33, "f32"), {"x": x.astype(np.float32)})["y"]
    sm = O.evaluate(softmax_graph(7, 33, "f32"), {"x": x.astype(np.float32)})["y"]
    np.testing.assert_allclose(np.exp(ls), sm, rtol=1e-13)
    np.testing.assert_allclose(np.exp(ls).sum(axis=-1), 1.0, rtol=1e-13)
    # brute force, python loops
    xr = x.astype(np.float32).astype(np.float64)
    for r in range(2):
        m = max(xr[r])
        want = [v - m - math.log(sum(math.exp(u - m) for u in xr[r])) for v in xr[r]]
        np.testing.assert_allclose(ls[r], want, rtol=1e-13, atol=1e-13)


def test_max_rel_err_metric():
    ref = np.array([1.0, 0.0, -2.0, 1e-9])
    got = np.array([1.001, 0.0, -2.0, 2e-9])
    assert O.max_rel_err(got, ref) == pytest.approx(1.0)             # tiny element dominates when strict
    assert O.max_rel_err(got, ref, floor=O.rms(ref)) == pytest.approx(0.001 / O.rms(ref), rel=1e-6)
    assert O.max_rel_err(np.zeros(3), np.zeros(3)) == 0.0
