"""The comparison rule of tests/parity.py, exercised on the CPU with hand-made "device" outputs.

What is checked: (1) the graph rewrite that lets the oracle take the device's bf16 roundings,
(2) that a one-step difference in a computed bf16 node passes while everything downstream is still
held to the fp32 tolerance, (3) the conditioning mask from the fp64 companion run.
"""
import numpy as np
import pytest

import oracle
from parity import Reference, check_all, check_output, expose_bf16_nodes, forced_graph, quantiser_nodes
from workloads import Graph, bf16_bits_to_f32, f32_to_bf16_bits


def _round_trip_graph(rows, cols):
    g = Graph()
    x = g.input(rows, cols, name="x")
    c = g.input(rows, cols, name="c")
    s = g.unary("sigmoid", x, name="s")
    q = g.unary("convert", s, "bf16", name="q")
    f = g.unary("convert", q, "f32", name="f")
    t = g.unary("tanh", f, name="t")
    d = g.binary("sub", t, c, name="d")
    g.set_outputs([d])
    return g, q


def test_quantiser_nodes_and_exposure():
    g, q = _round_trip_graph(4, 8)
    assert quantiser_nodes(g) == [q]
    with pytest.raises(AssertionError):
        Reference(g, [])           # consumed bf16 node that is not a plan output
    e = expose_bf16_nodes(g)
    assert e.outputs == g.outputs + [q] and g.outputs == [6]   # a copy: the original is untouched
    # bf16 inputs and unconsumed bf16 outputs are not quantisers
    h = Graph()
    i = h.input(2, 2, "bf16")
    h.set_outputs([h.unary("convert", h.unary("neg", h.unary("convert", i, "f32")), "bf16")])
    assert quantiser_nodes(h) == []


def test_forced_graph_structure():
    g, q = _round_trip_graph(4, 8)
    g = expose_bf16_nodes(g)
    g2, computed, forced_input = forced_graph(g, [q])
    assert len(g2.nodes) == len(g.nodes) + 1
    fin = forced_input[q]
    assert g2.nodes[fin].op == "input" and g2.nodes[fin].dtype == "bf16"
    assert g2.nodes[computed[q]].op == "convert" and g2.nodes[computed[q]].dtype == "bf16"
    # the consumer of q reads the stand-in; q itself is still computed from its own operand
    f2 = next(i for i, n in enumerate(g2.nodes) if n.name == "f")
    assert g2.nodes[f2].ins == (fin,)
    assert g2.outputs == [computed[o] for o in g.outputs]
    assert all(o < i for i, n in enumerate(g2.nodes) for o in n.ins)   # still topological
    # forcing the oracle's own values changes nothing
    rng = np.random.default_rng(5)
    ins = [rng.standard_normal((4, 8)).astype(np.float32), rng.standard_normal((4, 8)).astype(np.float32)]
    a = oracle.run(g, ins, 1)
    a2 = oracle.run(g2, [ins[0], ins[1], a[1]], 1)
    np.testing.assert_array_equal(a2[0], a[0])
    np.testing.assert_array_equal(a2[1], a[1])


def _device_like(ins, flip_at=None):
    """What a correct device could return for _round_trip_graph: q may sit one bf16 step off at `flip_at`."""
    x, c = ins
    s = (1.0 / (1.0 + np.exp(-x.astype(np.float64)))).astype(np.float32)
    q = f32_to_bf16_bits(s)
    if flip_at is not None:
        q = q.copy()
        q[flip_at] += 1          # the neighbouring bf16 value (positive numbers: one step up)
    t = np.tanh(bf16_bits_to_f32(q).astype(np.float64)).astype(np.float32)
    return [(t.astype(np.float64) - c).astype(np.float32), q]


def test_a_one_step_difference_in_a_bf16_node_is_shared_not_forgiven():
    rows, cols = 16, 64
    g = expose_bf16_nodes(_round_trip_graph(rows, cols)[0])
    rng = np.random.default_rng(7)
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    # at one element c nearly equals tanh(sigmoid(x)): the subtraction cancels there, so a bf16 step upstream is
    # amplified far beyond the fp32 tolerance (which is relative to the tensor's rms, ~0.3)
    scale = 1 + 0.5 * rng.standard_normal((rows, cols))
    scale[3, 17] = 1 + 1e-3
    c = (np.tanh(1.0 / (1.0 + np.exp(-x.astype(np.float64)))) * scale).astype(np.float32)
    ins = [x, c]
    ref = Reference(g, ins, threads=2)
    check_all(g, _device_like(ins), ref, "no flip")
    flipped = _device_like(ins, flip_at=(3, 17))
    check_all(g, flipped, ref, "one bf16 step at one element")
    # without sharing the rounding that element is far outside the fp32 tolerance (this is what the old blanket slack hid)
    with pytest.raises(AssertionError):
        check_output(flipped[0], ref.a[0], "f32", "plain comparison")
    # sharing the rounding forgives nothing downstream ...
    bad = [flipped[0].copy(), flipped[1]]
    bad[0][3, 17] += np.float32(3e-5)
    with pytest.raises(AssertionError):
        check_all(g, bad, ref, "downstream error")
    # ... and a bf16 node that is more than a rounding step away from the oracle's still fails
    far = _device_like(ins)
    far[1] = far[1].copy()
    far[1][5, 5] += 4
    with pytest.raises(AssertionError):
        check_all(g, far, ref, "four bf16 steps")


def test_conditioning_mask_from_the_fp64_companion():
    rows, cols = 8, 512
    g = Graph()
    u, v = g.input(rows, cols), g.input(rows, cols)
    g.set_outputs([g.binary("sub", g.unary("exp", u), g.unary("exp", v))])
    rng = np.random.default_rng(11)
    uu = rng.uniform(-1, 1, (rows, cols)).astype(np.float32)
    vv = rng.uniform(-1, 1, (rows, cols)).astype(np.float32)
    # one element: the difference of two values near e^12, each rounded to fp32 first (absolute error ~1e-2)
    uu[2, 100], vv[2, 100] = np.float32(12.0), np.float32(12.0 - 3e-5)
    ref = Reference(g, [uu, vv], threads=2)
    a, b = ref.a[0], ref.b[0]
    gap = abs(float(a[2, 100]) - float(b[2, 100]))
    assert gap > 1e-4                        # ill-conditioned by construction
    st = check_all(g, [b], ref, "device = the fp64 companion")
    assert st[0]["ill_conditioned"] == 1
    # the mask is not a free pass: the element is still held to a multiple of the A-B gap
    dev = a.copy()
    dev[2, 100] += np.float32(40 * gap + 1.0)
    with pytest.raises(AssertionError):
        check_all(g, [dev], ref, "far off at the ill-conditioned element")
    # and a well-conditioned element gets no slack from it
    dev = a.copy()
    dev[0, 0] += np.float32(1e-3)
    with pytest.raises(AssertionError):
        check_all(g, [dev], ref, "error at a well-conditioned element")
    # too many ill-conditioned elements is itself a failure (the workload would not test anything)
    uu2, vv2 = uu.copy(), vv.copy()
    uu2[:, :64] = np.float32(12.0)
    vv2[:, :64] = np.float32(12.0 - 3e-5)
    ref2 = Reference(g, [uu2, vv2], threads=2)
    with pytest.raises(AssertionError):
        check_all(g, [ref2.a[0]], ref2, "an eighth of the tensor ill-conditioned")


def test_accumulation_companion_flags_cancelling_sums():
    # tanh(row sum): for a row whose 5000 terms cancel to ~0.05 the fp32 sum is uncertain by ~1e-5 in ANY order, and tanh
    # passes that on at slope 1, while the other rows (|sum| ~ 40) are saturated and insensitive.  The fp64-throughout
    # companion does not see this (the summands are the same to 1e-7); the accumulation companion does.
    rows, cols = 64, 5000
    g = Graph()
    x = g.input(rows, cols)
    g.set_outputs([g.unary("tanh", g.reduce_row("sum", g.unary("tanh", x)))])
    rng = np.random.default_rng(3)
    xv = rng.standard_normal((rows, cols)).astype(np.float32)
    t = np.tanh(xv.astype(np.float64)).astype(np.float32).astype(np.float64)
    for r in (0, 1):   # make the rows' sums 0.05 by bending one element (arctanh of what is missing)
        rest = 0.05 - (t[r].sum() - t[r, -1])
        while abs(rest) >= 0.99:   # spread over more elements when one cannot carry it
            xv[r, np.argmax(np.sign(rest) * -t[r])] = np.float32(2.0 * np.sign(rest))
            t[r] = np.tanh(xv[r].astype(np.float64)).astype(np.float32)
            rest = 0.05 - (t[r].sum() - t[r, -1])
        xv[r, -1] = np.float32(np.arctanh(rest))
    ref = Reference(g, [xv], threads=2)
    assert abs(float(np.arctanh(ref.a[0][0, 0])) - 0.05) < 1e-3
    # a device that sums in fp32 in another order (numpy's pairwise float32 sum)
    s32 = np.tanh(xv.astype(np.float64)).astype(np.float32).sum(axis=1, dtype=np.float32, keepdims=True)
    dev = np.tanh(s32.astype(np.float64)).astype(np.float32)
    st = check_all(g, [dev], ref, "pairwise fp32 sum")
    assert st[0]["ill_conditioned"] >= 2
    assert np.abs(ref.b[0] - ref.a[0]).max() < 2e-6 < np.abs(ref.c[0] - ref.a[0])[:2].max()   # B is blind to it, C is not
    # the flagged rows are still bounded by a multiple of the companion's gap, the others by the plain tolerance
    bad = dev.copy()
    bad[0, 0] += np.float32(0.05)
    with pytest.raises(AssertionError):
        check_all(g, [bad], ref, "far off on a flagged row")
    bad = dev.copy()
    bad[40, 0] -= np.float32(1e-3)
    with pytest.raises(AssertionError):
        check_all(g, [bad], ref, "off on a saturated row")


def test_spread_flags_what_one_realisation_of_the_noise_can_miss():
    # max over a row of differences of nearly equal tanh values: results ~1e-4 from operands ~0.5.  Whether |A - B| at an element
    # is large is a matter of luck (how close the fp32 roundings of the two tanh values came to their fp64 values); the spread S is
    # not: every element of this output is flagged, and a device that is one operand spacing off passes, while it would not on a
    # well-conditioned output, and ten times that still fails here.
    rows, cols = 200, 64
    g = Graph()
    ia, ib = g.input(rows, cols), g.input(rows, cols)
    g.set_outputs([g.reduce_row("max", g.binary("sub", g.unary("tanh", ia), g.unary("tanh", ib))), g.unary("tanh", ia)])
    rng = np.random.default_rng(11)
    a = rng.uniform(0.3, 1.0, (rows, cols)).astype(np.float32)
    b = (a - rng.uniform(0, 2e-4, (rows, cols)).astype(np.float32)).astype(np.float32)
    ref = Reference(g, [a, b], threads=2)
    tol = 1e-5 * np.abs(ref.a[0]) + 1e-5 * float(np.sqrt(np.mean(ref.a[0].astype(np.float64) ** 2)))
    lucky = np.abs(ref.b[0].astype(np.float64) - ref.a[0]) < 0.25 * tol
    assert lucky.any() and (ref.s[0] > tol).all()          # B alone would leave some elements unflagged; S flags them all
    dev = [ref.a[0].copy(), ref.a[1].copy()]
    i = int(np.argmax(lucky))
    dev[0][i, 0] += np.float32(6e-8)                       # one spacing of a value in [0.5, 1)
    st = check_all(g, dev, ref, "one operand spacing off", max_ill_fraction=0.5)
    assert st[0]["ill_conditioned"] == rows and st[1]["ill_conditioned"] == 0
    dev[0][i, 0] += np.float32(5e-6)
    with pytest.raises(AssertionError):
        check_all(g, dev, ref, "far beyond the spread", max_ill_fraction=0.5)
    dev = [ref.a[0].copy(), ref.a[1].copy()]
    dev[1][3, 5] += np.float32(1e-4)                      # the well-conditioned output gets no slack
    with pytest.raises(AssertionError):
        check_all(g, dev, ref, "off on a well-conditioned output", max_ill_fraction=0.5)
