"""Pins of the CPU oracle against things other than itself.

The paper prints no worked numerical example, so nothing here comes from paper-printed
values; the oracle is pinned by closed forms, invariants, pure-Python brute force,
numpy.float32 bit equality for the correctly rounded ops, and torch CPU fp64 library
routines (softmax, layer_norm, gelu).  A planted mistake (dropped term, swapped operand,
wrong reduce axis, wrong rounding) fails at least one test below.
"""
import decimal
import math
import os
import sys

import numpy as np
import pytest
import torch

import oracle
from workloads import (Graph, bf16_bits_to_f32, f32_to_bf16_bits, layernorm_gelu_graph, multi_reduce_graph,
                       softmax_graph, elementwise20_graph, elementwise20_inputs, random_dag_graph,
                       random_dag_inputs)

RNG = np.random.default_rng(12345)


def run1(g, ins, **kw):
    return oracle.run(g, ins, **kw)


def unary_graph(op, rows, cols, dtype="f32"):
    g = Graph()
    x = g.input(rows, cols, dtype)
    g.set_outputs([g.unary(op, x)])
    return g


def binary_graph(op, rows, cols):
    g = Graph()
    a = g.input(rows, cols)
    b = g.input(rows, cols)
    g.set_outputs([g.binary(op, a, b)])
    return g


# ------------------------------------------------------------------ roundings
def test_round_f32_is_numpy_cast():
    xs = np.concatenate([RNG.standard_normal(2000) * 10.0 ** RNG.integers(-40, 38, 2000),
                         [0.0, -0.0, 1.0 + 2.0 ** -24, 1.0 + 2.0 ** -24 + 2.0 ** -50, 1e-45, 3e38 * 1.2]])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float32).astype(np.float64)
    for x, w in zip(xs, want):
        assert oracle.round_f32(x) == w or (math.isinf(w) and math.isinf(oracle.round_f32(x)))


def test_round_bf16_matches_torch_and_generator():
    xs = np.concatenate([RNG.standard_normal(4000) * 10.0 ** RNG.integers(-30, 30, 4000),
                         # ties: exactly halfway between two bf16 values -> even
                         [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8),
                          2.0 ** -126, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -133, 2.0 ** -127 * 1.01, 3.38e38, 3.4e38]])
    # torch narrows fp64 -> fp32 -> bf16 (two roundings); feed it fp32-representable values so both
    # routes are a single rounding
    xs = xs.astype(np.float32).astype(np.float64)
    t = torch.from_numpy(xs).to(torch.bfloat16).double().numpy()
    got = np.array([oracle.round_bf16(x) for x in xs])
    np.testing.assert_array_equal(got, t)
    # the input generator's fp32->bf16 (bit trick) agrees on fp32 values
    f = xs.astype(np.float32)
    f = f[np.isfinite(f)]
    np.testing.assert_array_equal(bf16_bits_to_f32(f32_to_bf16_bits(f)).astype(np.float64),
                                  np.array([oracle.round_bf16(float(v)) for v in f]))
    # closed form: 1 + 2^-8 ties to 1 (even), 1 + 3*2^-8 ties to 1 + 2^-6
    assert oracle.round_bf16(1.0 + 2.0 ** -8) == 1.0
    assert oracle.round_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    # a single rounding from fp64: just above the tie goes up (a route through fp32 would lose the 2^-40)
    assert oracle.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 1.0 + 2.0 ** -7


# ------------------------------------------------------------------ elementwise ops
PY_UNARY = {
    "neg": lambda x: -x, "abs": abs, "exp": math.exp, "log": math.log, "tanh": math.tanh,
    "sigmoid": lambda x: math.exp(x) / (1.0 + math.exp(x)),          # a different algebraic form
    "sqrt": lambda x: x ** 0.5, "rsqrt": lambda x: x ** -0.5, "rcp": lambda x: x ** -1.0,
    "gelu_tanh": lambda x: 0.5 * x * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3))),
}


@pytest.mark.parametrize("op", sorted(PY_UNARY))
def test_unary_brute_force(op):
    x = RNG.uniform(0.1, 4.0, (3, 7)).astype(np.float32)
    if op not in ("log", "sqrt", "rsqrt", "rcp"):
        x *= RNG.choice([-1.0, 1.0], x.shape).astype(np.float32)
    got = run1(unary_graph(op, 3, 7), [x])[0]
    for i in range(3):
        for j in range(7):
            want = PY_UNARY[op](float(x[i, j]))
            assert got[i, j] == pytest.approx(want, rel=2e-7, abs=1e-38), (op, x[i, j])


def _dec_tanh(d):
    e2 = (2 * d).exp()
    return (e2 - 1) / (e2 + 1)


DEC_UNARY = {   # 40-digit decimal arithmetic: no code in common with the C math library the oracle calls
    "exp": lambda d: d.exp(), "log": lambda d: d.ln(), "tanh": _dec_tanh, "sigmoid": lambda d: 1 / (1 + (-d).exp()),
    "gelu_tanh": lambda d: d / 2 * (1 + _dec_tanh((decimal.Decimal(2) / decimal.Decimal("3.14159265358979323846264338327950288")).sqrt()
                                                  * (d + decimal.Decimal("0.044715") * d ** 3))),
}


@pytest.mark.parametrize("op", sorted(DEC_UNARY))
def test_transcendentals_vs_decimal_arithmetic(op):
    # test_unary_brute_force goes through the same libm as the oracle for exp / log / tanh; this one does not
    decimal.getcontext().prec = 40
    x = np.concatenate([RNG.uniform(-8, 8, 24), [0.0, 1e-6, -1e-6, 0.25, -0.25, 20.0, -20.0]]).astype(np.float32).reshape(1, -1)
    if op == "log":
        x = np.abs(x) + np.float32(1e-3)
    if op == "gelu_tanh":   # below -5 the definition 0.5 z (1 + tanh u) cancels even in fp64: the oracle, which IS the definition, loses digits
        x = np.maximum(x, np.float32(-5.0))
    got = run1(unary_graph(op, *x.shape), [x])[0]
    for j in range(x.shape[1]):
        want = float(DEC_UNARY[op](decimal.Decimal(float(x[0, j]))))
        assert got[0, j] == pytest.approx(want, rel=1.2e-7, abs=1e-38), (op, x[0, j])   # half an fp32 ulp + the cast


def test_unary_identities():
    x = RNG.uniform(-5, 5, (4, 8)).astype(np.float32)
    t = run1(unary_graph("tanh", 4, 8), [x])[0]
    tn = run1(unary_graph("tanh", 4, 8), [-x])[0]
    np.testing.assert_array_equal(t, -tn)                      # odd
    s = run1(unary_graph("sigmoid", 4, 8), [x])[0].astype(np.float64)
    sn = run1(unary_graph("sigmoid", 4, 8), [-x])[0].astype(np.float64)
    np.testing.assert_allclose(s + sn, 1.0, atol=1.2e-7)       # sigma(x)+sigma(-x)=1
    th = run1(unary_graph("tanh", 4, 8), [x / 2])[0].astype(np.float64)
    np.testing.assert_allclose(s, 0.5 * (1 + th), atol=1.2e-7)  # sigma(x) = (1+tanh(x/2))/2
    g = run1(unary_graph("gelu_tanh", 1, 4), [np.array([[0.0, 30.0, -30.0, 1e-3]], np.float32)])[0]
    assert g[0, 0] == 0.0 and g[0, 1] == 30.0 and abs(g[0, 2]) == 0.0
    # torch library routine in fp64
    z = torch.from_numpy(x).double()
    want = torch.nn.functional.gelu(z, approximate="tanh").float().numpy()
    np.testing.assert_array_equal(run1(unary_graph("gelu_tanh", 4, 8), [x])[0], want)
    # exp(log x) = x
    p = np.abs(x) + 0.5
    g2 = Graph()
    i = g2.input(4, 8)
    g2.set_outputs([g2.unary("exp", g2.unary("log", i))])
    np.testing.assert_allclose(run1(g2, [p])[0], p, rtol=3e-7)


@pytest.mark.parametrize("op,npop", [("add", np.add), ("sub", np.subtract), ("mul", np.multiply),
                                     ("div", np.divide), ("max", np.maximum), ("min", np.minimum)])
def test_binary_bit_equal_to_numpy_float32(op, npop):
    a = (RNG.standard_normal((5, 33)) * 10.0 ** RNG.integers(-3, 4, (5, 33))).astype(np.float32)
    b = (RNG.standard_normal((5, 33)) * 10.0 ** RNG.integers(-3, 4, (5, 33))).astype(np.float32)
    got = run1(binary_graph(op, 5, 33), [a, b])[0]
    np.testing.assert_array_equal(got.view(np.uint32), npop(a, b).astype(np.float32).view(np.uint32))


def test_sqrt_bit_equal_to_numpy_float32():
    a = np.abs(RNG.standard_normal((3, 50)) * 1e3).astype(np.float32)
    np.testing.assert_array_equal(run1(unary_graph("sqrt", 3, 50), [a])[0], np.sqrt(a))


def test_cmp_select_truth_table():
    a = np.array([[1.0, 2.0, 2.0, -0.0, 0.0, -3.0]], np.float32)
    b = np.array([[2.0, 1.0, 2.0, 0.0, -0.0, -3.5]], np.float32)
    want = {"gt": [0, 1, 0, 0, 0, 1], "ge": [0, 1, 1, 1, 1, 1], "lt": [1, 0, 0, 0, 0, 0],
            "le": [1, 0, 1, 1, 1, 0], "eq": [0, 0, 1, 1, 1, 0], "ne": [1, 1, 0, 0, 0, 1]}
    for kind, w in want.items():
        g = Graph()
        ia, ib = g.input(1, 6), g.input(1, 6)
        p = g.cmp(kind, ia, ib)
        s = g.select(p, ia, ib)
        g.set_outputs([p, s])
        pm, sel = run1(g, [a, b])
        assert pm.dtype == np.uint8 and pm[0].tolist() == w, kind
        np.testing.assert_array_equal(sel.view(np.uint32), np.where(np.array(w, bool), a, b).view(np.uint32))


def test_u8_plan_input_through_select_truth_table():
    # a predicate tensor that enters the plan from outside: any non-zero byte selects the first branch (bits of the
    # chosen operand, signed zeros and all); hand-written expectations, no library routine in between
    p = np.array([[0, 1, 2, 255, 0, 1], [1, 0, 0, 128, 7, 0]], np.uint8)
    a = np.array([[1.5, -2.0, 3.25, -0.0, 0.0, 1e-30], [7.0, 8.0, 9.0, 10.0, -11.0, 12.0]], np.float32)
    b = np.array([[-1.5, 2.0, -3.25, 0.0, -0.0, -1e30], [-7.0, -8.0, -9.0, -10.0, 11.0, -12.0]], np.float32)
    want = np.array([[-1.5, -2.0, 3.25, -0.0, -0.0, 1e-30], [7.0, -8.0, -9.0, 10.0, -11.0, -12.0]], np.float32)
    g = Graph()
    ip, ia, ib = g.input(2, 6, "u8"), g.input(2, 6), g.input(2, 6)
    s = g.select(ip, ia, ib)
    g.set_outputs([s, g.select(ip, ib, ia)])
    got, swapped = run1(g, [p, a, b])
    np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
    np.testing.assert_array_equal(swapped.view(np.uint32), np.where(want.view(np.uint32) == a.view(np.uint32), b, a).view(np.uint32))
    # the predicate bytes themselves pass through a transpose unchanged in meaning (normalised to 0/1)
    g2 = Graph()
    ip2 = g2.input(2, 6, "u8")
    g2.set_outputs([g2.transpose(ip2)])
    np.testing.assert_array_equal(run1(g2, [p])[0], (p.T != 0).astype(np.uint8))
    # bf16 branches: the chosen operand's bf16 bits
    g3 = Graph()
    jp, ja, jb = g3.input(1, 4, "u8"), g3.input(1, 4, "bf16"), g3.input(1, 4, "bf16")
    g3.set_outputs([g3.select(jp, ja, jb)])
    abits = np.array([[0x3F80, 0xBF80, 0x0000, 0x8000]], np.uint16)
    bbits = np.array([[0x4000, 0xC000, 0x8000, 0x0000]], np.uint16)
    np.testing.assert_array_equal(run1(g3, [np.array([[1, 0, 0, 9]], np.uint8), abits, bbits])[0],
                                  np.array([[0x3F80, 0xC000, 0x8000, 0x8000]], np.uint16))


def test_convert_and_bf16_nodes():
    x = RNG.standard_normal((4, 16)).astype(np.float32)
    g = Graph()
    i = g.input(4, 16, "f32")
    c = g.unary("convert", i, "bf16")
    back = g.unary("convert", c, "f32")
    sq = g.binary("mul", c, c, "bf16")   # bf16 node: fp32-exact product rounded once to bf16
    g.set_outputs([c, back, sq])
    cb, bk, sqb = run1(g, [x])
    t = torch.from_numpy(x).to(torch.bfloat16)
    np.testing.assert_array_equal(bf16_bits_to_f32(cb), t.float().numpy())
    np.testing.assert_array_equal(bk, t.float().numpy())
    prod = (t.double() * t.double()).to(torch.bfloat16)
    np.testing.assert_array_equal(bf16_bits_to_f32(sqb), prod.float().numpy())


# ------------------------------------------------------------------ shape ops
def test_transpose_broadcast_index_rules():
    x = np.arange(3 * 5, dtype=np.float32).reshape(3, 5)
    g = Graph()
    i = g.input(3, 5)
    t = g.transpose(i)
    tt = g.transpose(t)
    g.set_outputs([t, tt])
    tr, back = run1(g, [x])
    for r in range(3):
        for c in range(5):
            assert tr[c, r] == x[r, c]
    np.testing.assert_array_equal(back, x)
    # broadcasts: explicit index rule, then reduce back = N * v
    v = np.arange(1, 6, dtype=np.float32).reshape(1, 5)
    w = np.arange(1, 4, dtype=np.float32).reshape(3, 1)
    g = Graph()
    iv, iw, ix = g.input(1, 5), g.input(3, 1), g.input(3, 5)
    bv = g.binary("add", ix, g.bcast_rowvec(iv, 3))
    bw = g.binary("add", ix, g.bcast_colvec(iw, 5))
    zero = g.binary("sub", ix, ix)
    cv = g.reduce_col("sum", g.binary("add", zero, g.bcast_rowvec(iv, 3)))
    rw = g.reduce_row("sum", g.binary("add", zero, g.bcast_colvec(iw, 5)))
    g.set_outputs([bv, bw, cv, rw])
    o_bv, o_bw, o_cv, o_rw = run1(g, [v, w, x])
    for r in range(3):
        for c in range(5):
            assert o_bv[r, c] == x[r, c] + v[0, c]
            assert o_bw[r, c] == x[r, c] + w[r, 0]
    np.testing.assert_array_equal(o_cv, 3 * v)
    np.testing.assert_array_equal(o_rw, 5 * w)


# ------------------------------------------------------------------ reductions
@pytest.mark.parametrize("kind", ["sum", "max", "min", "mean"])
def test_reductions_vs_fsum_and_numpy(kind):
    x = (RNG.standard_normal((6, 37)) * 100).astype(np.float32)
    g = Graph()
    i = g.input(6, 37)
    g.set_outputs([g.reduce_row(kind, i), g.reduce_col(kind, i)])
    rr, rc = run1(g, [x])
    assert rr.shape == (6, 1) and rc.shape == (1, 37)
    py = {"sum": math.fsum, "max": max, "min": min, "mean": lambda v: math.fsum(v) / len(v)}[kind]
    for r in range(6):
        assert rr[r, 0] == np.float32(py([float(t) for t in x[r]]))
    for c in range(37):
        assert rc[0, c] == np.float32(py([float(t) for t in x[:, c]]))


def test_accumulation_companion_displaces_sums_by_one_rounding_unit_per_term():
    # round_nodes=2: sum (and the sum inside a mean) + 2^-24 * sum |terms|, then the usual rounding; max / min and
    # everything that is not a reduction are untouched.  Closed forms first, then numpy in fp64.
    g = Graph()
    i = g.input(1, 4)
    g.set_outputs([g.reduce_row("sum", i), g.reduce_row("mean", i)])
    s, m = run1(g, [np.array([[1.0, -1.0, 0.5, 0.0]], np.float32)], round_nodes=2)
    # sum 0.5, sum |terms| 2.5: 0.5 + 2.5 * 2^-24 lies half-way between two floats (spacing 2^-24 there) -> the even one
    assert float(s[0, 0]) == 0.5 + 2 * 2.0 ** -24 and float(m[0, 0]) == np.float32((0.5 + 2.5 * 2.0 ** -24) / 4)
    s, _ = run1(g, [np.array([[3.0, 3.0, 3.0, 3.0]], np.float32)], round_nodes=2)
    assert float(s[0, 0]) == 12.0 + 2.0 ** -20    # positive terms: a relative 2^-24 = 0.75 of the spacing at 12, rounds up one step
    x = (RNG.standard_normal((7, 1001)) * 10.0 ** RNG.integers(-2, 3, (7, 1001))).astype(np.float32)
    g = Graph()
    i = g.input(7, 1001)
    g.set_outputs([g.reduce_row("sum", i), g.reduce_col("sum", i), g.reduce_row("mean", i), g.reduce_col("mean", i),
                   g.reduce_row("max", i), g.reduce_col("min", i), g.unary("tanh", i)])
    rs, cs, rm, cm, mx, mn, th = run1(g, [x], round_nodes=2)
    x64 = x.astype(np.float64)
    for axis, got_s, got_m, n in ((1, rs, rm, 1001), (0, cs, cm, 7)):
        want = np.array([math.fsum(v) + math.fsum(abs(t) for t in v) * 2.0 ** -24 for v in (x64 if axis == 1 else x64.T)])
        np.testing.assert_allclose(got_s.ravel(), want, rtol=1.2e-7)
        np.testing.assert_allclose(got_m.ravel(), want / n, rtol=1.2e-7)
    ref = run1(g, [x])
    np.testing.assert_array_equal(mx, ref[4])
    np.testing.assert_array_equal(mn, ref[5])
    np.testing.assert_array_equal(th, ref[6])


def test_spread_companion_against_numpy_float32_arithmetic():
    # round_nodes=3 returns no values but the first-order spread of a correct fp32 implementation around the reference.  It is
    # pinned against such implementations: numpy's own float32 arithmetic (correctly rounded + - * /, a float32 tanh, a pairwise
    # float32 sum), whose actual deviation from the fp64 result must be of the size the spread says - within 4.5 spreads almost
    # everywhere (rounding noise enters as a standard deviation, the error of an approximated op as one spacing), and neither far
    # below nor far above it in the root mean square.
    n = 20000
    x, y, z, w = (RNG.uniform(-2, 2, (1, n)).astype(np.float32) for _ in range(4))
    g = Graph()
    ix, iy, iz, iw = (g.input(1, n) for _ in range(4))
    chain = g.binary("sub", g.binary("mul", g.binary("add", g.binary("mul", ix, iy), iz), iw), g.binary("div", ix, g.binary("add", g.unary("abs", iy), g.const(1.0, 1, n))))
    g.set_outputs([chain])
    sd = run1(g, [x, y, z, w], round_nodes=3)[0]
    assert sd.dtype == np.float64 and sd.shape == (1, n)
    f32 = ((x * y + z) * w - x / (np.abs(y) + np.float32(1.0))).astype(np.float32)   # every op rounded to float32 by numpy
    x64, y64, z64, w64 = (v.astype(np.float64) for v in (x, y, z, w))
    err = np.abs(f32.astype(np.float64) - ((x64 * y64 + z64) * w64 - x64 / (np.abs(y64) + 1.0)))
    ratio = err / sd
    assert (ratio < 4.5).mean() > 0.999 and 0.3 < np.sqrt(np.mean(ratio ** 2)) < 1.5, (ratio.max(), np.sqrt(np.mean(ratio ** 2)))
    # a difference of nearly equal tanh values: results ~1e-3 from operands ~0.5, each carrying one float32 tanh error
    g = Graph()
    ix, iy = g.input(1, n), g.input(1, n)
    g.set_outputs([g.binary("sub", g.unary("tanh", ix), g.unary("tanh", iy))])
    a = RNG.uniform(0.3, 1.0, (1, n)).astype(np.float32)
    b = (a + RNG.uniform(-1e-3, 1e-3, (1, n)).astype(np.float32)).astype(np.float32)
    sd = run1(g, [a, b], round_nodes=3)[0]
    f32 = (np.tanh(a) - np.tanh(b)).astype(np.float32)          # float32 tanh: within a spacing or so of the true value
    err = np.abs(f32.astype(np.float64) - (np.tanh(a.astype(np.float64)) - np.tanh(b.astype(np.float64))))
    ratio = err / sd
    assert (ratio < 4.5).mean() > 0.999 and 0.1 < np.sqrt(np.mean(ratio ** 2)) < 1.5, (ratio.max(), np.sqrt(np.mean(ratio ** 2)))
    assert np.median(sd / np.abs(f32.astype(np.float64) + 1e-30)) > 1e-5   # ... which is far more than 1e-5 of such a result
    # row sums of 4096 products of random sign, summed pairwise in float32 by numpy
    rows, cols = 512, 4096
    p, q = RNG.standard_normal((rows, cols)).astype(np.float32), RNG.standard_normal((rows, cols)).astype(np.float32)
    g = Graph()
    ip, iq = g.input(rows, cols), g.input(rows, cols)
    g.set_outputs([g.reduce_row("sum", g.binary("mul", ip, iq)), g.reduce_row("mean", g.binary("mul", ip, iq))])
    sd_sum, sd_mean = run1(g, [p, q], round_nodes=3)
    f32 = (p * q).sum(axis=1, dtype=np.float32, keepdims=True)
    exact = np.array([[math.fsum(float(u) * float(v) for u, v in zip(pr, qr))] for pr, qr in zip(p, q)])
    ratio = np.abs(f32.astype(np.float64) - exact) / sd_sum
    assert ratio.max() < 4.5 and 0.05 < np.sqrt(np.mean(ratio ** 2)) < 1.5, (ratio.max(), np.sqrt(np.mean(ratio ** 2)))
    assert (sd_mean >= sd_sum / cols).all() and (sd_mean < 1.5 * sd_sum / cols).all()   # the sum's spread over n, plus the division's own rounding


def test_spread_companion_structure():
    # what is exact has no spread; data movement carries the spread with the values; max / min and select carry the spread of
    # the element they pick
    rows, cols = 6, 10
    x = RNG.uniform(-1, 1, (rows, cols)).astype(np.float32)
    y = RNG.uniform(-1, 1, (rows, cols)).astype(np.float32)
    g = Graph()
    ix, iy = g.input(rows, cols), g.input(rows, cols)
    e = g.unary("exp", ix)
    pred = g.cmp("gt", ix, iy)
    g.set_outputs([g.unary("neg", ix), pred, g.select(pred, ix, iy), e, g.transpose(e), g.reshape(e, cols, rows), g.binary("max", e, iy),
                   g.select(pred, e, iy), g.reduce_row("max", e), g.concat(e, iy, "cols"), g.binary("add", e, g.bcast_colvec(g.reduce_row("max", e), cols))])
    neg, pr, sel_in, se, st, sr, smax, ssel, srmax, scat, sadd = run1(g, [x, y], round_nodes=3)
    assert not neg.any() and not pr.any() and not sel_in.any()           # inputs, predicates, moves of inputs: exact
    assert (se > 0).all() and (se < 1e-6).all()
    np.testing.assert_array_equal(st, se.T)
    np.testing.assert_array_equal(sr, se.reshape(cols, rows))
    ev = np.exp(x.astype(np.float64))
    np.testing.assert_array_equal(smax, np.where(ev.astype(np.float32) >= y, se, 0.0))
    np.testing.assert_array_equal(ssel, np.where(x > y, se, 0.0))
    np.testing.assert_array_equal(srmax[:, 0], se[np.arange(rows), np.argmax(x, axis=1)])   # exp is monotonic: the largest x
    np.testing.assert_array_equal(scat, np.concatenate([se, np.zeros_like(se)], axis=1))
    # the errors of two approximated results add linearly (they may lean the same way); the add's own rounding comes on top, in quadrature
    assert (sadd >= se + srmax).all() and (sadd < se + srmax + 3e-7).all()


def test_softmax_pins():
    R, C = 8, 1024
    g = softmax_graph(R, C)
    x = RNG.standard_normal((R, C)).astype(np.float32)
    y = run1(g, [x])[0]
    assert np.all(y > 0) and np.all(y <= 1)
    np.testing.assert_allclose(y.astype(np.float64).sum(1), 1.0, atol=C * 2.0 ** -24)
    # constant row -> exactly 1/C = 2^-10
    yc = run1(g, [np.full((R, C), 3.25, np.float32)])[0]
    assert np.all(yc == np.float32(2.0 ** -10))
    # shift invariance (shift exactly representable so x+c is exact for these x)
    xs = np.round(x * 256) / 256
    y1 = run1(g, [xs.astype(np.float32)])[0]
    y2 = run1(g, [(xs + 4.0).astype(np.float32)])[0]
    np.testing.assert_array_equal(y1, y2)
    # torch fp64 library softmax; fp64-through companion agrees to fp32 rounding
    want = torch.softmax(torch.from_numpy(x).double(), -1).numpy()
    yb = run1(g, [x], round_nodes=False)[0]
    np.testing.assert_array_equal(yb, want.astype(np.float32))
    np.testing.assert_allclose(y, want, rtol=4e-7)


def test_layernorm_pins():
    R, C = 16, 1024
    g = layernorm_gelu_graph(R, C)
    x = RNG.standard_normal((R, C)).astype(np.float32) * 3 + 1
    xb = f32_to_bf16_bits(x)
    gamma = RNG.normal(1, 0.1, (1, C)).astype(np.float32)
    beta = RNG.normal(0, 0.1, (1, C)).astype(np.float32)
    bias = RNG.normal(0, 0.02, (1, C)).astype(np.float32)
    out = bf16_bits_to_f32(run1(g, [xb, gamma, beta, bias])[0])
    xd = torch.from_numpy(bf16_bits_to_f32(xb)).double()
    ln = torch.nn.functional.layer_norm(xd, (C,), torch.from_numpy(gamma[0]).double(),
                                        torch.from_numpy(beta[0]).double(), 1e-5) + torch.from_numpy(bias).double()
    want = torch.nn.functional.gelu(ln, approximate="tanh")
    # within one bf16 ulp of the fp64 library result, and the fp64-through companion is its exact rounding
    np.testing.assert_allclose(out, want.numpy(), rtol=2.0 ** -7, atol=1e-6)
    outb = bf16_bits_to_f32(run1(g, [xb, gamma, beta, bias], round_nodes=False)[0])
    assert np.mean(outb != want.to(torch.bfloat16).float().numpy()) < 1e-3
    # decomposed GeLU agrees with the composite op
    gd = layernorm_gelu_graph(R, C, decomposed_gelu=True)
    outd = bf16_bits_to_f32(run1(gd, [xb, gamma, beta, bias])[0])
    np.testing.assert_allclose(outd, out, rtol=2.0 ** -7, atol=1e-6)

    # the normalisation alone: gamma=1, beta=0 -> row mean 0, variance var/(var+eps)
    g2 = Graph()
    xi = g2.input(R, C)
    mu = g2.reduce_row("mean", xi)
    xc = g2.binary("sub", xi, g2.bcast_colvec(mu, C))
    var = g2.reduce_row("mean", g2.binary("mul", xc, xc))
    rstd = g2.unary("rsqrt", g2.binary("add", var, g2.const(1e-5, R, 1)))
    xn = g2.binary("mul", xc, g2.bcast_colvec(rstd, C))
    g2.set_outputs([xn, var])
    xn_o, var_o = run1(g2, [x])
    np.testing.assert_allclose(xn_o.astype(np.float64).mean(1), 0.0, atol=1e-6)
    v = var_o.astype(np.float64)[:, 0]
    np.testing.assert_allclose(xn_o.astype(np.float64).var(1), v / (v + 1e-5), rtol=1e-5)
    # constant row -> exactly 0 after centring; scale invariance
    xn_c = run1(g2, [np.full((R, C), 2.5, np.float32)])[0]
    assert np.all(xn_c == 0)
    xn_s = run1(g2, [(x * 4).astype(np.float32)])[0]
    np.testing.assert_allclose(xn_s, xn_o, rtol=1e-4, atol=1e-5)


def test_backward_graphs_vs_torch_autograd():
    # the LayerNorm-backward and softmax-backward subgraphs against torch's fp64 autograd of the forward ops
    from workloads import layernorm_grad_graph, softmax_grad_graph
    R, C = 24, 96
    x = RNG.standard_normal((R, C)).astype(np.float32) * 2 + 0.5
    dy = RNG.standard_normal((R, C)).astype(np.float32)
    gamma = RNG.normal(1, 0.1, (1, C)).astype(np.float32)
    dx, dgamma, dbeta = run1(layernorm_grad_graph(R, C), [x, dy, gamma])
    xt = torch.from_numpy(x).double().requires_grad_()
    gt = torch.from_numpy(gamma[0]).double().requires_grad_()
    bt = torch.zeros(C, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.layer_norm(xt, (C,), gt, bt, 1e-5).backward(torch.from_numpy(dy).double())
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=2e-5, atol=2e-6)
    np.testing.assert_allclose(dgamma[0], gt.grad.numpy(), rtol=2e-5, atol=2e-5)
    np.testing.assert_allclose(dbeta[0], bt.grad.numpy(), rtol=2e-5, atol=2e-5)
    # dx is orthogonal to the constant vector and to xhat (the two projections the formula removes)
    assert np.abs(dx.astype(np.float64).sum(1)).max() < 1e-4

    z = RNG.standard_normal((R, C)).astype(np.float32)
    zt = torch.from_numpy(z).double().requires_grad_()
    yt = torch.softmax(zt, dim=1)
    yt.backward(torch.from_numpy(dy).double())
    y32 = yt.detach().float().numpy()
    (dz,) = run1(softmax_grad_graph(R, C), [y32, dy])
    np.testing.assert_allclose(dz, zt.grad.numpy(), rtol=1e-4, atol=1e-7)
    assert np.abs(dz.astype(np.float64).sum(1)).max() < 1e-6  # softmax gradients sum to zero over a row


def test_multi_reduce_pins():
    R, C = 64, 16
    g = multi_reduce_graph(R, C)
    cs, cq, rn = run1(g, [np.full((R, C), 0.5, np.float32)])
    assert np.all(cs == R * 0.5) and np.all(cq == R * 0.25) and np.all(rn == 0.5 * 4.0)
    x = RNG.normal(0.5, 1, (R, C)).astype(np.float32)
    cs, cq, rn = run1(g, [x])
    xd = x.astype(np.float64)
    np.testing.assert_array_equal(cs[0], xd.sum(0).astype(np.float32))
    np.testing.assert_allclose(cq[0], (xd * xd).sum(0), rtol=3e-7)
    np.testing.assert_allclose(rn[:, 0], np.sqrt((xd * xd).sum(1)), rtol=3e-7)
    # interchange of summation
    assert cq.astype(np.float64).sum() == pytest.approx((rn.astype(np.float64) ** 2).sum(), rel=1e-6)
    # non-square: a swapped axis would give the wrong shapes / values
    g = multi_reduce_graph(5, 512)
    cs, cq, rn = run1(g, [np.ones((5, 512), np.float32)])
    assert cs.shape == (1, 512) and rn.shape == (5, 1) and np.all(cs == 5) and np.all(rn == np.float32(math.sqrt(512)))


# ------------------------------------------------------------------ whole DAGs
_NP_UN = {"neg": np.negative, "abs": np.abs, "exp": np.exp, "log": np.log, "tanh": np.tanh,
          "sigmoid": lambda x: 1 / (1 + np.exp(-x)), "sqrt": np.sqrt, "rsqrt": lambda x: 1 / np.sqrt(x),
          "rcp": lambda x: 1 / x, "convert": lambda x: x}
_NP_BIN = {"add": np.add, "sub": np.subtract, "mul": np.multiply, "div": np.divide, "max": np.fmax, "min": np.fmin}
_NP_CMP = {"gt": np.greater, "ge": np.greater_equal, "lt": np.less, "le": np.less_equal, "eq": np.equal, "ne": np.not_equal}
_NP_RED = {"sum": np.sum, "max": np.max, "min": np.min, "mean": np.mean}


def numpy_eval(g, ins, order=None):
    """Independent vectorised evaluator (fp64 inside each op, one fp32 rounding per node)."""
    vals = {}
    it = iter(ins)
    for i in (order or range(len(g.nodes))):
        n = g.nodes[i]
        a = [vals[k] for k in n.ins]
        if n.op == "input":
            v = np.asarray(next(it) if order is None else ins[g.input_ids().index(i)], np.float64)
        elif n.op == "const":
            v = np.full((n.rows, n.cols), np.float32(n.value), np.float64)
        elif n.op in _NP_UN:
            v = _NP_UN[n.op](a[0])
        elif n.op in _NP_BIN:
            v = _NP_BIN[n.op](a[0], a[1])
        elif n.op == "cmp":
            v = _NP_CMP[n.attr](a[0], a[1]).astype(np.float64)
        elif n.op == "select":
            v = np.where(a[0] != 0, a[1], a[2])
        elif n.op == "bcast_rowvec" or n.op == "bcast_colvec":
            v = np.broadcast_to(a[0], (n.rows, n.cols))
        elif n.op == "transpose":
            v = a[0].T
        elif n.op == "reduce_row":
            v = _NP_RED[n.attr](a[0], axis=1, keepdims=True)
        elif n.op == "reduce_col":
            v = _NP_RED[n.attr](a[0], axis=0, keepdims=True)
        else:
            raise ValueError(n.op)
        vals[i] = v.astype(np.float32).astype(np.float64) if n.dtype == "f32" else v
    return [vals[o].astype(np.float32) if g.nodes[o].dtype == "f32" else vals[o].astype(np.uint8) for o in g.outputs]


def test_elementwise20_mask_and_values_vs_numpy():
    R = 64
    g = elementwise20_graph(R, 1024)
    ins = [a[:R] if a.shape[0] > 1 else a for a in elementwise20_inputs(R, 1024)]
    # expose the predicate too
    pid = next(i for i, n in enumerate(g.nodes) if n.op == "cmp")
    g.set_outputs(g.outputs + [pid])
    n17, n20, mask = run1(g, ins)
    a, b, c, _d, u, _v = ins
    want_mask = ((a + b).astype(np.float32) > (c * u).astype(np.float32)).astype(np.uint8)  # float32 ops
    np.testing.assert_array_equal(mask, want_mask)
    w17, w20, wm = numpy_eval(g, ins)
    np.testing.assert_array_equal(wm, mask)
    np.testing.assert_allclose(n17, w17, rtol=3e-7, atol=1e-30)
    np.testing.assert_allclose(n20, w20, rtol=3e-7, atol=2e-7)


def test_random_dag_vs_numpy_and_order_independence():
    g = random_dag_graph(num_nodes=120, rows=64, seed=7)
    ins = random_dag_inputs(g)
    got = run1(g, ins, num_threads=3)
    want = numpy_eval(g, ins)
    for a, b, o in zip(got, want, g.outputs):
        # sums are sequential fp64 in the oracle, pairwise in numpy: equal after fp32 rounding up to 1 ulp
        np.testing.assert_allclose(a, b, rtol=2.5e-7, atol=1e-30, err_msg=f"node {o}")
    # the oracle's result does not depend on the thread count
    again = run1(g, ins, num_threads=1)
    for a, b in zip(got, again):
        np.testing.assert_array_equal(a, b)


def _paper_figures():
    out = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_figures.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                out[line[0]] = float(line[1])
    return out


def test_e2e_formula_fixture():
    # Section 6.4: predicted end-to-end speedup = 1 + FusableRatio (1 - 1/FusionSpeedup).  With the printed geomean fusion
    # speedup and a fusable ratio inside the printed range the formula reproduces the printed ~13 % end-to-end figure, and over
    # the printed ranges it stays inside the printed 5-20 % band's order of magnitude.
    fig = _paper_figures()
    pred = 1 + 0.3 * (1 - 1 / fig["fusion_speedup_geomean"])
    assert pred == pytest.approx(1 + fig["e2e_speedup_geomean_pct"] / 100, abs=3e-3)
    lo = 1 + fig["fusable_ratio_min_pct"] / 100 * (1 - 1 / fig["fusion_speedup_min"])
    hi = 1 + fig["fusable_ratio_max_pct"] / 100 * (1 - 1 / fig["fusion_speedup_max"])
    assert 1.0 < lo < 1 + fig["e2e_speedup_min_pct"] / 100 < 1 + fig["e2e_speedup_max_pct"] / 100 < hi < 1.5


def test_oracle_reproduces_its_stored_small_cases():
    # tests/golden/oracle_small_cases.json was written by tests/golden/make_oracle_fixtures.py (oracle only): the oracle must
    # keep producing exactly those bits, and the softmax case is redone here by hand in fp64
    import json
    import math
    sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden"))
    import make_oracle_fixtures as mk
    stored = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "oracle_small_cases.json")))
    for name, g, ins in mk.cases():
        res = oracle.run(g, ins, 1)
        for r, hexes, shape in zip(res, stored[name]["outputs_hex"], stored[name]["output_shapes"]):
            got = (bf16_bits_to_f32(r) if r.dtype == np.uint16 else r.astype(np.float32)).view(np.uint32).ravel()
            assert list(r.shape) == shape and [format(int(v), "08x") for v in got] == hexes, name
    row = [0.0, 1.0, 2.0, 3.0]
    e = [math.exp(v - 3.0) for v in row]
    want = np.array([v / sum(e) for v in e], dtype=np.float64)
    got = np.array([int(h, 16) for h in stored["softmax_2x4"]["outputs_hex"][0][:4]], dtype=np.uint32).view(np.float32)
    np.testing.assert_allclose(got, want, rtol=2e-7)


# ------------------------------------------------------------------ reshape / bitcast / concat
def test_reshape_and_bitcast_keep_the_row_major_sequence():
    x = RNG.standard_normal((6, 20)).astype(np.float32)
    g = Graph()
    i = g.input(6, 20)
    a = g.reshape(i, 15, 8)
    b = g.reshape(a, 6, 20)                  # reshape o reshape^-1 = identity, bit for bit
    c = g.reshape(i, 1, 120, op="bitcast")
    d = g.view_nd(i, (2, 3, 4, 5), 3)        # [2,3,4,5] presented as [24, 5]
    e = g.view_nd(d, (2, 3, 4, 5), 1)        # ... and as [2, 60]
    g.set_outputs([a, b, c, d, e, g.unary("neg", a)])
    ra, rb, rc, rd, re_, rn = run1(g, [x])
    np.testing.assert_array_equal(rb.view(np.uint32), x.view(np.uint32))
    for got, shape in ((ra, (15, 8)), (rc, (1, 120)), (rd, (24, 5)), (re_, (2, 60))):
        assert got.shape == shape
        # brute force over flat indices: element k of the output is element k of the input
        for k in range(120):
            assert got[k // shape[1], k % shape[1]] == x[k // 20, k % 20]
    np.testing.assert_array_equal(rn, -x.reshape(15, 8))
    # an N-D softmax: [2,3,4,5] normalised over its last dim is the 2-D softmax of the [24,5] view
    g2 = Graph()
    j = g2.input(6, 20)
    v = g2.view_nd(j, (2, 3, 4, 5), 3)
    m = g2.reduce_row("max", v)
    ex = g2.unary("exp", g2.binary("sub", v, g2.bcast_colvec(m, 5)))
    y = g2.binary("div", ex, g2.bcast_colvec(g2.reduce_row("sum", ex), 5))
    g2.set_outputs([g2.reshape(y, 6, 20)])
    got = run1(g2, [x])[0]
    want = torch.softmax(torch.from_numpy(x).double().reshape(2, 3, 4, 5), dim=-1).reshape(6, 20).numpy()
    np.testing.assert_allclose(got, want, rtol=3e-7)
    # shape rule: the element count must not change
    g3 = Graph()
    k = g3.input(4, 4)
    r = g3.reshape(k, 2, 8)
    g3.nodes[r].cols = 7
    g3.set_outputs([r])
    with pytest.raises(RuntimeError):
        run1(g3, [np.zeros((4, 4), np.float32)])


def test_concat_index_rules_by_brute_force():
    a = RNG.standard_normal((5, 3)).astype(np.float32)
    b = RNG.standard_normal((5, 4)).astype(np.float32)
    c = RNG.standard_normal((2, 3)).astype(np.float32)
    g = Graph()
    ia, ib, ic = g.input(5, 3), g.input(5, 4), g.input(2, 3)
    cc = g.concat(ia, ib, "cols")
    cr = g.concat(ia, ic, "rows")
    g.set_outputs([cc, cr, g.reduce_row("sum", cc)])
    oc, orr, rs = run1(g, [a, b, c])
    assert oc.shape == (5, 7) and orr.shape == (7, 3)
    for i in range(5):
        for j in range(7):
            assert oc[i, j] == (a[i, j] if j < 3 else b[i, j - 3])
    for i in range(7):
        for j in range(3):
            assert orr[i, j] == (a[i, j] if i < 5 else c[i - 5, j])
    want = np.array([[math.fsum(map(float, a[i])) + math.fsum(map(float, b[i]))] for i in range(5)])
    np.testing.assert_allclose(rs, want, rtol=2e-7, atol=1e-7)
    # bf16 payloads are copied bit for bit
    g2 = Graph()
    ja, jb = g2.input(1, 2, "bf16"), g2.input(1, 3, "bf16")
    g2.set_outputs([g2.concat(ja, jb)])
    got = run1(g2, [np.array([[0x3F80, 0x8000]], np.uint16), np.array([[0x7F7F, 0x0001, 0xC000]], np.uint16)])[0]
    assert got.tolist() == [[0x3F80, 0x8000, 0x7F7F, 0x0001, 0xC000]]
    # shapes that do not add up are refused
    g3 = Graph()
    ka, kb = g3.input(2, 2), g3.input(2, 3)
    n = g3.concat(ka, kb)
    g3.nodes[n].cols = 6
    g3.set_outputs([n])
    with pytest.raises(RuntimeError):
        run1(g3, [np.zeros((2, 2), np.float32), np.zeros((2, 3), np.float32)])
