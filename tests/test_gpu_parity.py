"""GPU parity: the stitched kernels (through the C ABI) against the CPU oracle, element by element.

Tolerances (see tests/parity.py): fp32 outputs 1e-5, bf16 outputs 1e-2, predicates bit-exact.
Sizes span several workgroups, several loop trips and ragged tails; the five BASELINE workloads
are also checked at their full sizes in the launch configuration bench.py times.
"""
import os

import numpy as np
import pytest

import oracle
import paper_1811_05213_amd as fs
from paper_1811_05213_amd.runner import DeviceRun, run_graph
from parity import Reference, check_all, check_output, expose_bf16_nodes
from workloads import (Graph, bf16_bits_to_f32, elementwise20_graph, elementwise20_inputs, f32_to_bf16_bits,
                       layernorm_gelu_graph, layernorm_gelu_inputs, multi_reduce_graph, multi_reduce_inputs,
                       random_dag_graph, random_dag_inputs, softmax_graph, softmax_inputs, workload)

pytestmark = pytest.mark.gpu
RNG = np.random.default_rng(20240607)
THREADS = 16


def both_modes(g, ins, what, **kw):
    ref = Reference(g, ins)
    out_s = run_graph(g, ins, mode=fs.FS_MODE_STITCHED, **kw)
    check_all(g, out_s, ref, what + " stitched")
    out_u = run_graph(g, ins, mode=fs.FS_MODE_UNFUSED, **kw)
    check_all(g, out_u, ref, what + " unfused")
    return ref, out_s, out_u


# ------------------------------------------------------------------ single ops on awkward shapes
SHAPES = [(1, 1), (5, 3), (37, 1000), (300, 1), (1, 777), (64, 64), (129, 258), (2, 4100)]
UNARY_RANGES = {"neg": (-5, 5), "abs": (-5, 5), "exp": (-20, 20), "log": (1e-3, 50), "tanh": (-6, 6), "sigmoid": (-20, 20),
                "sqrt": (0, 100), "rsqrt": (1e-3, 100), "rcp": (0.01, 100), "gelu_tanh": (-8, 8)}


@pytest.mark.parametrize("op", sorted(UNARY_RANGES))
def test_unary_ops(op):
    lo, hi = UNARY_RANGES[op]
    for rows, cols in SHAPES:
        g = Graph()
        x = g.input(rows, cols)
        g.set_outputs([g.unary(op, x)])
        both_modes(g, [RNG.uniform(lo, hi, (rows, cols)).astype(np.float32)], f"{op} {rows}x{cols}")


@pytest.mark.parametrize("op", ["add", "sub", "mul", "div", "max", "min"])
def test_binary_ops_bit_exact(op):
    # correctly rounded IEEE ops: the GPU must agree with the oracle bit for bit
    for rows, cols in SHAPES[:6]:
        g = Graph()
        a, b = g.input(rows, cols), g.input(rows, cols)
        g.set_outputs([g.binary(op, a, b)])
        ins = [(RNG.standard_normal((rows, cols)) * 10.0 ** RNG.integers(-3, 4, (rows, cols))).astype(np.float32) for _ in range(2)]
        ref, out_s, out_u = both_modes(g, ins, f"{op} {rows}x{cols}")
        np.testing.assert_array_equal(out_s[0].view(np.uint32), ref[0].view(np.uint32))
        np.testing.assert_array_equal(out_u[0].view(np.uint32), ref[0].view(np.uint32))


def test_transcendental_accuracy_wide_range():
    """Pure relative error of the approximate ops over wide ranges (no rms slack): <= 1e-5."""
    cases = {"exp": np.linspace(-85, 85, 20001), "tanh": np.concatenate([np.linspace(-12, 12, 20001), np.logspace(-8, 0, 2000)]),
             "sigmoid": np.linspace(-30, 30, 20001), "log": np.logspace(-30, 30, 20001), "rsqrt": np.logspace(-30, 30, 20001),
             "rcp": np.logspace(-30, 30, 20001), # (the definition 0.5 z (1 + tanh u) cancels even in fp64 for z << -5: the oracle itself loses digits there)
             "gelu_tanh": np.concatenate([np.linspace(-5, 9, 20001), np.logspace(-8, 0, 2000)])}
    for op, xs in cases.items():
        x = xs.astype(np.float32).reshape(1, -1)
        g = Graph()
        i = g.input(*x.shape)
        g.set_outputs([g.unary(op, i)])
        ref = oracle.run(g, [x], THREADS)[0].astype(np.float64)
        out = run_graph(g, [x])[0].astype(np.float64)
        ok = np.abs(ref) > 1e-30
        rel = np.abs(out[ok] - ref[ok]) / np.abs(ref[ok])
        assert rel.max() <= 1e-5, f"{op}: max relative error {rel.max():.3g}"


def test_cmp_select_and_u8_outputs():
    rows, cols = 70, 300
    a = RNG.integers(-3, 4, (rows, cols)).astype(np.float32)  # many ties
    b = RNG.integers(-3, 4, (rows, cols)).astype(np.float32)
    for kind in ("gt", "ge", "lt", "le", "eq", "ne"):
        g = Graph()
        ia, ib = g.input(rows, cols), g.input(rows, cols)
        p = g.cmp(kind, ia, ib)
        s = g.select(p, ia, ib)
        g.set_outputs([p, s])
        ref, out_s, out_u = both_modes(g, [a, b], f"cmp {kind}")
        np.testing.assert_array_equal(out_s[0], ref[0])
        np.testing.assert_array_equal(out_s[1].view(np.uint32), ref[1].view(np.uint32))
    # a u8 tensor as plan input
    g = Graph()
    ip, ia, ib = g.input(rows, cols, "u8"), g.input(rows, cols), g.input(rows, cols)
    g.set_outputs([g.select(ip, ia, ib)])
    mask = RNG.integers(0, 2, (rows, cols)).astype(np.uint8)
    ref, out_s, _ = both_modes(g, [mask, a, b], "select with u8 input")
    np.testing.assert_array_equal(out_s[0], np.where(mask != 0, a, b))


def test_bf16_nodes_and_convert():
    rows, cols = 33, 520
    x = RNG.standard_normal((rows, cols)).astype(np.float32)
    g = Graph()
    i = g.input(rows, cols, "bf16")
    f = g.unary("convert", i, "f32")
    sq = g.binary("mul", i, i, "bf16")       # bf16 node kept in registers: rounded once
    y = g.binary("add", sq, f, "f32")
    o = g.unary("convert", y, "bf16")
    g.set_outputs([f, sq, y, o])
    ref, out_s, out_u = both_modes(g, [f32_to_bf16_bits(x)], "bf16 chain")
    # conversions and the exactly representable product are bit-exact
    np.testing.assert_array_equal(out_s[0], ref[0])
    np.testing.assert_array_equal(out_s[1], ref[1])


# ------------------------------------------------------------------ reductions, broadcasts, transposes
@pytest.mark.parametrize("kind", ["sum", "max", "min", "mean"])
def test_row_and_col_reductions(kind):
    for rows, cols in [(1, 1), (7, 5), (300, 1), (1, 777), (129, 258), (1000, 64), (40, 4100), (5000, 36)]:
        g = Graph()
        x = g.input(rows, cols)
        g.set_outputs([g.reduce_row(kind, x), g.reduce_col(kind, x)])
        both_modes(g, [RNG.standard_normal((rows, cols)).astype(np.float32)], f"reduce {kind} {rows}x{cols}")


def test_column_reductions_over_wide_rows():
    # wider than one workgroup's registers: column tiles, each with its own partials, tickets and fold
    for rows, cols in [(1000, 12288), (300, 100001), (5, 20000), (4097, 16384)]:
        g = Graph()
        x = g.input(rows, cols)
        g.set_outputs([g.reduce_col("sum", x), g.reduce_col("max", g.binary("mul", x, x)), g.reduce_col("mean", x)])
        p = fs.Plan(g)
        gi = p.group_info(0)
        assert gi["elems_per_lane"] * gi["lanes_per_row"] < cols
        if rows >= 300:  # (small launch-bound groups keep column folds apart)
            assert p.stats()["num_launches"] == 1 and gi["num_col_reduces"] == 3
        p.destroy()
        # (a mean away from zero: column sums of thousands of zero-mean terms cancel, and the rule would set such elements aside)
        both_modes(g, [(0.5 + RNG.standard_normal((rows, cols))).astype(np.float32)], f"wide column reductions {rows}x{cols}")
    # column tiles of 64 lanes from 513 columns on; bf16 rows are read 32 elements per lane; tiles that end inside a vector
    # and inside the row; per-column and per-row operands next to the reductions
    for rows, cols, dt in [(3000, 4096, "bf16"), (2200, 4104, "bf16"), (4100, 1030, "f32"), (900, 6152, "bf16"), (40, 2048, "f32")]:
        g = Graph()
        x = g.input(rows, cols, dt)
        b = g.input(1, cols)
        w = g.input(rows, 1)
        xf = g.unary("convert", x, "f32") if dt != "f32" else x
        y = g.binary("mul", g.binary("add", xf, g.bcast_rowvec(b, rows)), g.bcast_colvec(w, cols))
        g.set_outputs([g.reduce_col("sum", y), g.reduce_col("max", xf)])
        p = fs.Plan(g)
        gi = p.group_info(0)
        if rows >= 2000:  # (the smaller ones are launch-bound and keep their folds apart)
            assert p.stats()["num_launches"] == 1 and gi["lanes_per_row"] == 64 and gi["elems_per_lane"] == 4 * gi["vec_elems"]
        p.destroy()
        v = (0.5 + RNG.standard_normal((rows, cols))).astype(np.float32)
        ins = [f32_to_bf16_bits(v) if dt == "bf16" else v, RNG.standard_normal((1, cols)).astype(np.float32),
               (1.0 + RNG.random((rows, 1))).astype(np.float32)]
        both_modes(g, ins, f"column tiles {rows}x{cols} {dt}")
    # LayerNorm backward with a wide hidden dimension: the planner separates what cannot share a kernel
    g, ins, name = workload(6, 64)
    from workloads import layernorm_grad_graph, layernorm_grad_inputs
    g = layernorm_grad_graph(48, 16384)
    both_modes(g, layernorm_grad_inputs(48, 16384), "layernorm backward 48x16384")
    # row and column reductions over wide rows in one kernel: the in-workgroup column fold passes through LDS in pieces
    for rows, cols in ((3000, 4096), (700, 8200), (1500, 16384), (300, 30000)):
        g = layernorm_grad_graph(rows, cols)
        p = fs.Plan(g)
        assert p.stats()["num_launches"] == 1 and p.group_info(0)["lds_bytes"] <= 40000
        p.destroy()
        both_modes(g, layernorm_grad_inputs(rows, cols), f"layernorm backward {rows}x{cols}")
    g = multi_reduce_graph(2000, 8192)
    both_modes(g, multi_reduce_inputs(2000, 8192), "multi reduce 2000x8192")


def test_row_reduce_across_wavefronts():
    # rows long enough to be spread over 2..16 wavefronts with an LDS fold, ragged tails included
    for rows, cols in [(9, 4096), (3, 20000), (2, 16385), (5, 32768)]:  # 32768 = the longest row one workgroup holds
        g = softmax_graph(rows, cols)
        p = fs.Plan(g)
        assert p.group_info(0)["lanes_per_row"] > 64
        p.destroy()
        both_modes(g, [RNG.standard_normal((rows, cols)).astype(np.float32)], f"softmax {rows}x{cols}")


def test_rows_longer_than_a_workgroup_holds():
    # one workgroup per row walks it in column chunks, once per stage, recomputing what the stage needs (more than 32 rows
    # where the rows are beyond 256 KiB: fewer are cut into kernels that split the rows)
    for rows, cols in [(35, 100001), (33, 1 << 18), (1100, 40000), (300, 65536), (7, 50001), (34, 131072 + 4 * 77), (600, 32768)]:
        g = softmax_graph(rows, cols)
        p = fs.Plan(g)
        gi = p.group_info(0)
        assert p.stats()["num_launches"] == 1
        if cols % 4:  # (odd widths use scalar accesses: whichever form does not spill)
            pass
        elif cols <= 65536:  # up to 64 elements per lane of a 1024-lane workgroup still stay in registers (no spills: checked at plan creation)
            assert gi["elems_per_lane"] >= 32 and gi["elems_per_lane"] * gi["lanes_per_row"] >= cols
        else:  # longer: walked in chunks, the first 48 elements per lane resident
            assert gi["elems_per_lane"] == 48 and gi["elems_per_lane"] * gi["lanes_per_row"] < cols
        p.destroy()
        both_modes(g, [RNG.standard_normal((rows, cols)).astype(np.float32)], f"softmax {rows}x{cols}")
    # LayerNorm+bias+GeLU over bf16 rows: its three fp32 [1,C] operands outweigh the row, nothing stays resident in registers and
    # the row is kept in LDS as it came from memory (whole at 65544 columns, its first 160 KB at 100008)
    for rows, cols in [(35, 65544), (7, 40001), (34, 100008), (5, 65544)]:  # (the last: few rows, cut into kernels that split the rows)
        g = layernorm_gelu_graph(rows, cols)
        p = fs.Plan(g)
        gi = p.group_info(0)
        assert p.stats()["num_launches"] == 1 or rows <= 32
        if cols % 8 == 0 and rows > 32:
            assert gi["elems_per_lane"] == 16 and gi["lds_bytes"] > 2 * min(cols, 65536)
        p.destroy()
        both_modes(g, layernorm_gelu_inputs(rows, cols), f"layernorm+gelu {rows}x{cols}")
    # the same kernels under a caller's lanes-per-row hint: 512- and 256-lane workgroups walk more, shorter chunks
    for lanes in (512, 256):
        g = layernorm_gelu_graph(36, 65544)
        out = run_graph(g, layernorm_gelu_inputs(36, 65544), hint={"lanes_per_row": lanes})
        check_all(g, out, Reference(g, layernorm_gelu_inputs(36, 65544)), f"layernorm+gelu 36x65544, {lanes} lanes per row")
        g = softmax_graph(35, 100004)
        x = RNG.standard_normal((35, 100004)).astype(np.float32)
        check_all(g, run_graph(g, [x], hint={"lanes_per_row": lanes}), Reference(g, [x]), f"softmax 35x100004, {lanes} lanes per row")


def test_lds_buffered_results_on_long_rows():
    # rows beyond the registers with elementwise results kept in LDS between the passes (they take over the slot of the input they
    # dominate): fp32 softmax (exp), fp32 LayerNorm (x - mean), fp32 masked softmax (x * scale + mask, then exp); rows whose head only
    # fits the LDS run both forms of the last pass (read back below STAGE_CHUNKS, recomputed from memory beyond)
    from workloads.patterns import masked_softmax
    g = Graph()
    rows, cols = 40, 40000
    x, gam, bet = g.input(rows, cols), g.input(1, cols), g.input(1, cols)
    xc = g.binary("sub", x, g.bcast_colvec(g.reduce_row("mean", x), cols))
    rstd = g.unary("rsqrt", g.binary("add", g.reduce_row("mean", g.binary("mul", xc, xc)), g.const(1e-5, rows, 1)))
    g.set_outputs([g.binary("add", g.binary("mul", g.binary("mul", xc, g.bcast_colvec(rstd, cols)), g.bcast_rowvec(gam, rows)), g.bcast_rowvec(bet, rows))])
    p = fs.Plan(g)
    assert "sub (dominates it)" in p.group_source(0) and "if (ch < STAGE_CHUNKS) {" in p.group_source(0)
    p.destroy()
    ins = [(0.5 + RNG.standard_normal((rows, cols))).astype(np.float32), RNG.normal(1, .1, (1, cols)).astype(np.float32), RNG.normal(0, .1, (1, cols)).astype(np.float32)]
    both_modes(g, ins, "layernorm fp32 40x40000")
    for dt in ("f32", "bf16"):
        for rows, cols in ((36, 70000), (33, 131080)):
            g = masked_softmax(rows, cols, dt)
            v = [RNG.standard_normal((rows, cols)).astype(np.float32) * 4, np.where(RNG.random((rows, cols)) < 0.2, -30.0, 0.0).astype(np.float32)]
            both_modes(g, [f32_to_bf16_bits(a) if dt == "bf16" else a for a in v], f"masked softmax {dt} {rows}x{cols}")
    g = softmax_graph(40, 100000)
    x = RNG.standard_normal((40, 100000)).astype(np.float32)
    ref = Reference(g, [x])
    for budget in (0, 70000, 20000):  # all the LDS the device allows, a head of one chunk, no room for any chunk
        p = fs.Plan(g, lds_budget_bytes=budget)
        assert ("exp (dominates it)" in p.group_source(0)) == (budget != 20000)
        p.destroy()
        check_all(g, run_graph(g, [x], lds_budget_bytes=budget), ref, f"softmax 40x100000, LDS budget {budget}")


def test_broadcasts_and_transpose():
    rows, cols = 130, 72
    g = Graph()
    x, v, w = g.input(rows, cols), g.input(1, cols), g.input(rows, 1)
    a = g.binary("mul", x, g.bcast_rowvec(v, rows))
    b = g.binary("add", a, g.bcast_colvec(w, cols))
    c = g.binary("sub", b, g.const(0.25, rows, cols))
    t = g.transpose(c)
    tt = g.unary("tanh", t)          # consumer in the transposed space: next group
    r = g.reduce_row("sum", t)       # [cols,1]
    back = g.transpose(tt)
    g.set_outputs([c, t, tt, r, back])
    ins = [RNG.standard_normal((rows, cols)).astype(np.float32), RNG.standard_normal((1, cols)).astype(np.float32),
           RNG.standard_normal((rows, 1)).astype(np.float32)]
    ref, out_s, _ = both_modes(g, ins, "bcast/transpose")
    np.testing.assert_array_equal(out_s[1], out_s[0].T)  # a transpose moves bits, nothing else


def test_vector_valued_members_and_constants():
    # ops on [1,C] and [R,1] tensors inside a group with [R,C] work
    rows, cols = 90, 200
    g = Graph()
    x, v = g.input(rows, cols), g.input(1, cols)
    v2 = g.binary("mul", v, g.const(2.0, 1, cols))          # per-column value computed once per workgroup
    m = g.reduce_row("max", x)
    m2 = g.binary("add", m, g.const(1.0, rows, 1))          # per-row value
    y = g.binary("div", g.binary("add", x, g.bcast_rowvec(v2, rows)), g.bcast_colvec(m2, cols))
    g.set_outputs([y, v2, m2])
    ins = [RNG.uniform(1, 2, (rows, cols)).astype(np.float32), RNG.uniform(1, 2, (1, cols)).astype(np.float32)]
    both_modes(g, ins, "vector members")


# ------------------------------------------------------------------ the five workloads
@pytest.mark.parametrize("cfg,rows", [(1, 256), (1, 33), (1, 5000), (2, 512), (2, 77), (3, 256), (3, 1001), (4, 512), (4, 5000),
                                      (4, 70001), (5, None), (5, 100), (6, 777), (6, 4096), (7, 1000)])
def test_workloads_test_sizes(cfg, rows):
    g, ins, name = workload(cfg, rows)
    both_modes(g, ins, name)


def test_backward_subgraphs_are_one_kernel():
    # LayerNorm backward: four row reductions in three stages and two column reductions, one launch
    for cfg in (6, 7):
        g, _, _ = workload(cfg, 2048)
        p = fs.Plan(g)
        assert p.stats()["num_launches"] == 1
        p.destroy()


def test_layernorm_decomposed_gelu_variant():
    g = layernorm_gelu_graph(300, 1024, decomposed_gelu=True)
    ins = layernorm_gelu_inputs(300, 1024)
    ref, out_s, _ = both_modes(g, ins, "layernorm decomposed gelu")
    g2 = layernorm_gelu_graph(300, 1024)
    out2 = run_graph(g2, ins)
    check_output(out_s[0], out2[0], "bf16", "decomposed vs composite gelu")


def test_full_size_softmax_layernorm_multireduce_randomdag():
    for cfg in (1, 2, 4, 5):
        g, ins, name = workload(cfg)
        ref = Reference(g, ins)
        out = run_graph(g, ins)
        check_all(g, out, ref, name + " full size")


def test_full_size_elementwise20_on_sampled_rows():
    # every op of workload 3 is row-independent, so the oracle evaluated on a sample of rows gives
    # the exact expected values of those rows of the full-size run
    rows, cols = 65536, 1024
    g = elementwise20_graph(rows, cols)
    ins = elementwise20_inputs(rows, cols)
    out = run_graph(g, ins)
    pick = np.unique(np.concatenate([[0, 1, 255, 256, rows - 2, rows - 1], RNG.integers(0, rows, 500)]))
    gs = elementwise20_graph(len(pick), cols)
    ref = Reference(gs, [a[pick] if a.shape[0] == rows else a for a in ins])
    check_all(gs, [o[pick] for o in out], ref, "elementwise20 full size, sampled rows")
    assert all(np.isfinite(o).all() for o in out)


def test_tensors_beyond_two_to_the_31_elements_on_sampled_rows():
    # 2.16e9 elements (8.7 GB) per tensor: element indices and byte offsets past 32 bits.  The input is drawn on the
    # device (seeded); the oracle evaluates a sample of rows, which is exact because every op here is row-independent.
    import torch
    rows, cols = (1 << 21) + 3, 1032

    def build(r):
        g = Graph()
        x = g.input(r, cols)
        y = g.binary("mul", g.unary("tanh", x), x)
        g.set_outputs([y, g.reduce_row("sum", y), g.binary("sub", y, g.bcast_colvec(g.reduce_row("max", x), cols))])
        return g
    g = build(rows)
    plan = fs.Plan(g)
    assert plan.stats()["num_launches"] == 1
    r = DeviceRun(plan)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(181105213)
    x = torch.empty((rows, cols), dtype=torch.float32, device="cuda:0").uniform_(-2, 2, generator=gen)
    r.set_device_inputs([x])
    r.launch()
    torch.cuda.synchronize()
    pick = np.unique(np.concatenate([[0, 1, (1 << 20) - 1, 1 << 20, (1 << 21) - 1, 1 << 21, rows - 1], RNG.integers(0, rows, 300)]))
    idx = torch.from_numpy(pick).to("cuda:0")
    xs = x[idx].cpu().numpy()
    ref = Reference(build(len(pick)), [xs])
    got = [t[idx].cpu().numpy() for t in r.outputs]
    check_all(build(len(pick)), got, ref, "2^31+ elements, sampled rows")
    plan.destroy()


def test_elementwise20_predicate_bit_exact():
    rows = 300
    g = elementwise20_graph(rows, 1024)
    pid = next(i for i, n in enumerate(g.nodes) if n.op == "cmp")
    g.set_outputs(g.outputs + [pid])
    ins = elementwise20_inputs(rows, 1024)
    ref, out_s, out_u = both_modes(g, ins, "elementwise20 + mask")
    np.testing.assert_array_equal(out_s[2], ref[2])
    np.testing.assert_array_equal(out_u[2], ref[2])


def test_ragged_rows_with_staged_vectors_and_bf16():
    # LayerNorm chain on C not a multiple of the lane tiling (ragged vector indices), bf16 in/out:
    # exercises the LDS-staged per-column vectors with clamped lanes
    # (768, 384 and 192 bf16 columns: the lane count the row fills exactly, several rows per wavefront with 24 elements per lane)
    for rows, cols in ((300, 1000), (64, 520), (1000, 72), (5000, 768), (3001, 384), (7000, 192)):
        g = layernorm_gelu_graph(rows, cols)
        x = RNG.standard_normal((rows, cols)).astype(np.float32)
        ins = [f32_to_bf16_bits(x)] + [RNG.normal(m, s, (1, cols)).astype(np.float32) for m, s in ((1, .1), (0, .1), (0, .02))]
        both_modes(g, ins, f"layernorm {rows}x{cols}")


def test_looping_workgroups_with_operands_staged_once():
    # row-reduction groups with per-column operands whose workgroups loop and stage the operands in LDS once, before the loop:
    # row counts that are no multiple of the rows per trip (masked rows in the last trip), one-wavefront rows (16 rows per
    # trip), rows across 4 wavefronts, exact-fit lane counts (768 bf16 columns: 32 lanes x 3 vectors), a light operand
    from paper_1811_05213_amd import Plan
    from workloads import patterns as survey
    # (one-wavefront rows with up to four trips per workgroup ask for a trip's rows ahead: the first before the staging, the
    # next at the end of a trip -- [12301,1024]: workgroups with one and with two trips, [30011,1024]: three and four)
    for rows, cols in ((16391, 1024), (8197, 4096), (32771, 768), (12301, 1024), (30011, 1024), (40003, 1024)):
        g = layernorm_gelu_graph(rows, cols)
        p = Plan(g)
        gi = p.group_info(0)
        assert gi["grid"] * gi["rows_per_iter"] < rows and "fs_stage_rowvec" in p.group_source(0), (rows, cols, gi)
        assert ("row_first" in p.group_source(0)) == (cols <= 1024 and rows < 40000), (rows, cols)
        p.destroy()
        x = RNG.standard_normal((rows, cols)).astype(np.float32)
        ins = [f32_to_bf16_bits(x)] + [RNG.normal(m, s, (1, cols)).astype(np.float32) for m, s in ((1, .1), (0, .1), (0, .02))]
        both_modes(g, ins, f"looping layernorm {rows}x{cols}")
    g = survey.rmsnorm(8195, 2048)
    p = Plan(g)
    assert p.group_info(0)["grid"] * p.group_info(0)["rows_per_iter"] < 8195
    p.destroy()
    ins = [f32_to_bf16_bits(RNG.standard_normal((8195, 2048)).astype(np.float32)), RNG.normal(1, .1, (1, 2048)).astype(np.float32)]
    both_modes(g, ins, "looping rmsnorm 8195x2048")
    # the same schedule forced onto a small problem by hint: more workgroups than row tiles, workgroups without a trip
    g = layernorm_gelu_graph(50, 1024)
    x = RNG.standard_normal((50, 1024)).astype(np.float32)
    ins = [f32_to_bf16_bits(x)] + [RNG.normal(m, s, (1, 1024)).astype(np.float32) for m, s in ((1, .1), (0, .1), (0, .02))]
    ref = Reference(g, ins)
    for hint in ({"wg_threads": 1024, "max_workgroups": 2}, {"wg_threads": 1024, "max_workgroups": 512}, {"wg_threads": 256, "max_workgroups": 3}):
        check_all(g, run_graph(g, ins, hint=hint), ref, f"looping layernorm 50x1024 {hint}")


def test_unrolled_row_loop():
    # looping (column-reduction) kernels with two and three row tiles per trip
    g, ins, name = workload(4, 5000)
    ref = Reference(g, ins)
    for u in (2, 3):
        out = run_graph(g, ins, hint={"max_workgroups": 7, "tiles_per_trip": u})
        check_all(g, out, ref, f"{name} unroll {u}")


# ------------------------------------------------------------------ determinism and schedule invariance
def test_run_to_run_bit_identical():
    for cfg, rows in ((4, 70001), (1, 5000), (5, None)):
        g, ins, name = workload(cfg, rows)
        plan = fs.Plan(g)
        r = DeviceRun(plan)
        r.set_inputs(ins)
        r.launch()
        first = [o.copy() for o in r.results()]
        for _ in range(20):
            r.launch()
        for a, b in zip(first, r.results()):
            assert a.tobytes() == b.tobytes(), name
        plan.destroy()


def test_workspace_reuse_with_new_inputs():
    # the same plan and the same workspace (partials, tickets, tensors between groups) run on changing inputs: nothing of an
    # earlier run may be picked up by a later one (partials of the grid-wide folds are read with device-coherent loads, tickets
    # return to zero).  Column reductions, rows split over workgroups, the 200-node DAG, the few-long-rows softmax (3 kernels).
    cases = [workload(4, 70001)[:2], workload(6, 3000)[:2], workload(5)[:2], (softmax_graph(4, 300001), None)]
    g = Graph()
    x = g.input(3, 2100000)
    g.set_outputs([g.unary("sqrt", g.reduce_row("sum", g.binary("mul", x, x))), g.reduce_row("max", x)])
    cases.append((g, None))
    for g, ins in cases:
        plan = fs.Plan(g)
        r = DeviceRun(plan)
        for trial in range(4):
            rng = np.random.default_rng(9000 + trial)
            cur = []
            for k, i in enumerate(g.input_ids()):
                n = g.nodes[i]
                if ins is not None and trial == 0:
                    cur.append(ins[k])
                    continue
                a = rng.standard_normal((n.rows, n.cols)).astype(np.float32)  # (fresh draws of the distribution the graphs are built for)
                cur.append(f32_to_bf16_bits(a) if n.dtype == "bf16" else a)
            r.set_inputs(cur)
            r.launch()
            r.launch()
            check_all(g, r.results(), Reference(g, cur), f"workspace reuse, trial {trial}")
        plan.destroy()


@pytest.mark.parametrize("cfg,rows", [(1, 300), (2, 300), (4, 3000), (3, 200)])
def test_schedule_invariance(cfg, rows):
    """The one-block schedule (Section 4.3) and other legal schedules give the tuned schedule's result."""
    g, ins, name = workload(cfg, rows)
    ref = Reference(g, ins)
    for hint in ({"max_workgroups": 1}, {"lanes_per_row": 256, "wg_threads": 256}, {"lanes_per_row": 1024, "wg_threads": 1024},
                 {"lanes_per_row": 32, "wg_threads": 64, "max_workgroups": 7}, {"wg_threads": 512, "max_workgroups": 40}):
        out = run_graph(g, ins, hint=hint)
        check_all(g, out, ref, f"{name} hint {hint}")


def test_caller_given_groups():
    g = softmax_graph(200, 512)
    ins = softmax_inputs(200, 1024)[0][:, :512].copy()
    ref = Reference(g, [ins])
    grp = [0] * len(g.nodes)
    for k, i in enumerate(g.compute_ids()):
        grp[i] = [0, 1, 1, 2, 3][k]
    out = run_graph(g, [ins], group_of_node=grp)
    check_all(g, out, ref, "softmax in four caller-given groups")


# ------------------------------------------------------------------ run-time argument errors (nothing is launched)
def test_run_argument_errors():
    g, ins, _ = workload(4, 512)
    plan = fs.Plan(g)
    r = DeviceRun(plan)
    r.set_inputs(ins)
    need = plan.workspace_bytes()
    assert need > 0
    ptrs_in = [t.data_ptr() for t in r.inputs]
    ptrs_out = [t.data_ptr() for t in r.outputs]
    with pytest.raises(fs.FsError) as e:
        plan.run(ptrs_in, ptrs_out, 0, 0)
    assert e.value.status_name == "FS_ERR_WORKSPACE"
    with pytest.raises(fs.FsError) as e:
        plan.run(ptrs_in, ptrs_out, r.workspace.data_ptr(), need - 1)
    assert e.value.status_name == "FS_ERR_WORKSPACE"
    with pytest.raises(fs.FsError) as e:
        plan.run([ptrs_in[0] + 4], ptrs_out, r.workspace.data_ptr(), need)
    assert e.value.status_name == "FS_ERR_INVALID_ARG"
    # real device buffers that overlap: the row-norm output laid over the input, and over the workspace
    with pytest.raises(fs.FsError) as e:
        plan.run(ptrs_in, [ptrs_out[0], ptrs_out[1], ptrs_in[0] + 1024], r.workspace.data_ptr(), need)
    assert e.value.status_name == "FS_ERR_INVALID_ARG" and "overlaps inputs[0]" in str(e.value)
    with pytest.raises(fs.FsError) as e:
        plan.run(ptrs_in, [r.workspace.data_ptr(), ptrs_out[1], ptrs_out[2]], r.workspace.data_ptr(), need)
    assert e.value.status_name == "FS_ERR_INVALID_ARG" and "overlaps the workspace" in str(e.value)
    plan.load()   # explicit load: the first run after it allocates nothing
    plan.load()   # idempotent
    plan.workspace_check(r.workspace.data_ptr(), need)   # initialised by DeviceRun: clean
    r.launch()  # still usable afterwards
    check_all(g, r.results(), Reference(g, ins), "after argument errors")
    plan.workspace_check(r.workspace.data_ptr(), need)   # every run leaves the tickets at zero
    # a workspace that was never initialised (recycled memory) is reported, not silently mis-folded
    import torch
    dirty = torch.full((max(need, 256),), 0x5A, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(fs.FsError) as e:
        plan.workspace_check(dirty.data_ptr(), need)
    assert e.value.status_name == "FS_ERR_WORKSPACE" and "ticket" in str(e.value)
    plan.workspace_init(dirty.data_ptr(), need)
    plan.workspace_check(dirty.data_ptr(), need)
    lim = fs.device_limits()
    assert lim["from_device"] and lim["compute_units"] >= 1 and lim["lds_bytes_per_workgroup"] >= 65536
    plan.destroy()


def test_plans_replay_correctly_from_a_hip_graph():
    # fs_plan_run enqueues kernel launches only (no memset node, no allocation once the plan is loaded), so a caller may
    # capture it.  Every replay must reproduce the eager result bit for bit, with eager work and synchronisation in
    # between, also for plans with ticketed folds (the tickets return to zero inside each replay) and several kernels.
    import torch
    for cfg, rows in ((4, 3000), (5, None), (6, 700)):
        g, ins, name = workload(cfg, rows)
        plan = fs.Plan(g)
        r = DeviceRun(plan)
        r.set_inputs(ins)
        plan.load()
        r.launch()
        eager = [t.clone() for t in r.outputs]
        torch.cuda.synchronize()
        check_all(g, r.results(), Reference(g, ins), name + " eager")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            r.launch()
        for rep in range(4):
            for t in r.outputs:
                t.zero_()
            r2 = DeviceRun(plan)          # eager work of the same plan on other buffers between the replays
            r2.set_inputs(ins)
            r2.launch()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for k, (a, b) in enumerate(zip(r.outputs, eager)):
                assert torch.equal(a, b), f"{name}: replay {rep} output {k} differs from the eager run"
            for k, (a, b) in enumerate(zip(r2.outputs, eager)):
                assert torch.equal(a, b), f"{name}: eager run between replays, output {k}"
        del graph
        plan.destroy()


def test_transposes_through_lds_tile_and_direct():
    # tile path (several shapes, ragged rows/cols, bf16 and u8 payloads) and the direct path (forced by a tiny LDS budget)
    for rows, cols, dt in ((512, 256, "f32"), (130, 72, "f32"), (1000, 36, "f32"), (77, 200, "bf16"), (64, 4100, "f32"), (300, 1, "f32"), (1, 300, "f32")):
        g = Graph()
        x = g.input(rows, cols, dt)
        y = g.unary("neg", x)
        t = g.transpose(y)
        g.set_outputs([t, y])
        v = RNG.standard_normal((rows, cols)).astype(np.float32)
        ins = [f32_to_bf16_bits(v) if dt == "bf16" else v]
        for budget in (0, 64):
            ref = Reference(g, ins)
            out = run_graph(g, ins, lds_budget_bytes=budget)
            check_all(g, out, ref, f"transpose {rows}x{cols} {dt} budget {budget}")
            np.testing.assert_array_equal(out[0], out[1].T)
    # a predicate tensor, transposed
    g = Graph()
    a, b = g.input(90, 40), g.input(90, 40)
    g.set_outputs([g.transpose(g.cmp("gt", a, b))])
    ins = [RNG.standard_normal((90, 40)).astype(np.float32) for _ in range(2)]
    out = run_graph(g, ins)
    np.testing.assert_array_equal(out[0], (ins[0] > ins[1]).astype(np.uint8).T)


def test_very_narrow_rows():
    # rows of a few elements: one lane per row (no cross-lane step), odd widths with scalar accesses, per-column operands
    for rows, cols in ((100003, 3), (50000, 7), (30000, 13), (70000, 2), (65537, 8), (40000, 6), (9, 5)):
        g = Graph()
        x, w = g.input(rows, cols), g.input(1, cols)
        xs = g.binary("mul", x, g.bcast_rowvec(w, rows))
        n = g.unary("rsqrt", g.binary("add", g.reduce_row("sum", g.binary("mul", xs, xs)), g.const(1e-6, rows, 1)))
        y = g.binary("mul", xs, g.bcast_colvec(n, cols))
        g.set_outputs([y, g.reduce_row("max", y), g.reduce_row("mean", x)])
        ins = [RNG.standard_normal((rows, cols)).astype(np.float32), RNG.uniform(0.5, 2, (1, cols)).astype(np.float32)]
        both_modes(g, ins, f"narrow rows {rows}x{cols}")
        both_modes(softmax_graph(rows, cols), [ins[0]], f"narrow softmax {rows}x{cols}")


def test_few_very_long_rows_reduced_by_segments():
    # a handful of rows of millions of elements whose only results are per-row values: every row is cut into segments, one
    # workgroup each, and the segment results meet through the ticketed fold (several reductions, values before and after
    # them, a per-row and a per-column operand, bf16 payload, ragged last chunk and last segment)
    from paper_1811_05213_amd import Plan
    for rows, cols, dt in ((4, (1 << 22) + 3, "f32"), (1, 3000001, "f32"), (7, 1 << 20, "bf16"), (64, 262144 + 8, "f32"), (3, 2100000, "f32")):
        g = Graph()
        x = g.input(rows, cols, dt)
        w = g.input(rows, 1)
        b = g.input(1, cols)
        xf = g.unary("convert", x, "f32") if dt != "f32" else x
        xs = g.binary("add", g.binary("mul", xf, g.bcast_colvec(g.unary("tanh", w), cols)), g.bcast_rowvec(b, rows))
        ss = g.reduce_row("sum", g.binary("mul", xs, xs))
        mx = g.reduce_row("max", xs)
        mean = g.reduce_row("mean", xf)
        norm = g.unary("sqrt", ss)
        g.set_outputs([norm, mx, g.binary("div", mean, g.binary("add", norm, w)), g.reduce_row("min", xs)])
        p = Plan(g)
        assert p.stats()["num_launches"] == 1 and p.group_info(0)["grid"] > rows, (rows, cols, p.group_info(0))
        xv = (0.5 + RNG.standard_normal((rows, cols))).astype(np.float32)  # a mean well away from zero: no cancellation
        ins = [f32_to_bf16_bits(xv) if dt == "bf16" else xv, RNG.uniform(0.5, 2, (rows, 1)).astype(np.float32), (0.1 * RNG.standard_normal((1, cols))).astype(np.float32)]
        both_modes(g, ins, f"segmented rows {rows}x{cols} {dt}")
        both_modes(g, ins, f"segmented rows again {rows}x{cols} {dt}")  # the tickets are left at zero
    # [R,C] and [1,C] results that need no reduction result are stored by the segment workgroups
    for rows, cols in ((3, 700001), (20, 70000)):
        g = Graph()
        x, b = g.input(rows, cols), g.input(1, cols)
        xs = g.binary("mul", x, g.bcast_rowvec(b, rows))
        g.set_outputs([g.unary("tanh", xs), g.reduce_row("max", xs), g.unary("abs", b), g.unary("rsqrt", g.reduce_row("sum", g.binary("mul", xs, xs)))])
        p = Plan(g)
        assert "fs_store_row" in p.group_source(0) and p.group_info(0)["grid"] > rows
        ins = [RNG.standard_normal((rows, cols)).astype(np.float32), RNG.uniform(-2, 2, (1, cols)).astype(np.float32)]
        both_modes(g, ins, f"segmented rows with full outputs {rows}x{cols}")
    # groups that cannot take that form over up to 32 such rows are cut into ones that can: softmax and LayerNorm+GeLU
    for rows, cols in ((8, (1 << 20) + 5), (1, 1 << 21), (32, 70000)):
        g = softmax_graph(rows, cols)
        assert Plan(g).stats()["num_launches"] == 3
        both_modes(g, [RNG.standard_normal((rows, cols)).astype(np.float32)], f"few long rows softmax {rows}x{cols}")
    g = layernorm_gelu_graph(3, 300000)
    assert Plan(g).stats()["num_launches"] > 1
    both_modes(g, layernorm_gelu_inputs(3, 300000), "few long rows LayerNorm+GeLU")
    # the layered planner takes the same cut; a caller's own plan (the whole softmax as one group) is honoured and runs as
    # one kernel that walks each row in chunks
    g = softmax_graph(4, 300001)
    x = RNG.standard_normal((4, 300001)).astype(np.float32)
    ref = Reference(g, [x])
    check_all(g, run_graph(g, [x], mode=fs.FS_MODE_LAYERED), ref, "few long rows softmax, layered planner")
    one = [0 if n.op not in ("input", "const", "bcast_rowvec", "bcast_colvec") else -1 for n in g.nodes]
    p = Plan(g, group_of_node=one)
    assert p.stats()["num_launches"] == 1 and p.group_info(0)["grid"] == 4
    p.destroy()
    check_all(g, run_graph(g, [x], group_of_node=one), ref, "few long rows softmax, caller's single group")


def test_wide_transposes_in_2d_tiles():
    # reduction-free groups with transposed roots over more than 256 columns: 2-D tiles through LDS (ragged in both directions,
    # bf16 and u8 payloads, several roots, per-column and per-row operands)
    # (tiles are walked in bands of column tiles when a row has more tiles than a band: full bands, ragged last bands of
    # 1, 15 and 24 tiles, one and several row tiles; the narrower shapes have too few column tiles for bands)
    for rows, cols, dt in ((300, 5000, "f32"), (5, 300, "f32"), (3, 70001, "f32"), (7000, 258, "bf16"), (1031, 1030, "f32"), (64, 4100, "f32"),
                           (2100, 3000, "bf16")):
        g = Graph()
        x = g.input(rows, cols, dt)
        b = g.input(1, cols)
        w = g.input(rows, 1)
        xf = g.unary("convert", x, "f32") if dt != "f32" else x
        y = g.binary("mul", g.binary("add", xf, g.bcast_rowvec(b, rows)), g.bcast_colvec(w, cols))
        yo = g.unary("convert", y, dt) if dt != "f32" else y
        t = g.transpose(yo)
        m = g.transpose(g.cmp("gt", y, xf))
        g.set_outputs([t, yo, m, g.transpose(g.unary("neg", xf))])
        p = fs.Plan(g)
        src = p.group_source(0)
        assert p.stats()["num_launches"] == 1 and p.group_info(0)["lds_bytes"] > 0
        assert ("in_band" in src) == (cols > 2100) and ("it % CT" in src) != ("in_band" in src)
        p.destroy()
        v = RNG.standard_normal((rows, cols)).astype(np.float32)
        ins = [f32_to_bf16_bits(v) if dt == "bf16" else v, RNG.standard_normal((1, cols)).astype(np.float32),
               RNG.standard_normal((rows, 1)).astype(np.float32)]
        ref, out_s, _ = both_modes(g, ins, f"tiled transpose {rows}x{cols} {dt}")
        np.testing.assert_array_equal(out_s[0], out_s[1].T)
        np.testing.assert_array_equal(out_s[2], ref[2])


def test_values_recomputed_by_the_kernels_that_need_them():
    # an elementwise value needed on both sides of a kernel boundary is computed on both sides instead of stored and read:
    # batch normalisation (the centred values), with a third reader and with the value kept as a plan output; a chain of
    # producers that spans two kernels (a bf16 input's conversion, the centring) or one (the exponentials of a softmax over a
    # handful of very long rows)
    from workloads.patterns import batchnorm
    for rows, cols in ((3000, 520), (20000, 1024), (700, 4100)):
        g = batchnorm(rows, cols)
        p = fs.Plan(g)
        if rows * cols * 4 >= (16 << 20):  # (smaller ones are launch-bound and keep their column folds apart: other kernels)
            assert p.stats()["num_launches"] == 3 and p.workspace_bytes() < rows * cols * 4
        p.destroy()
        ins = [(0.5 + RNG.standard_normal((rows, cols))).astype(np.float32), RNG.standard_normal((1, cols)).astype(np.float32),
               RNG.standard_normal((1, cols)).astype(np.float32)]
        both_modes(g, ins, f"batchnorm {rows}x{cols}")
    for kw in ({"extra_reader": True}, {"keep_as_output": True}):
        rows, cols = 5000, 1032
        g = Graph()
        x = g.input(rows, cols, "bf16")
        xf = g.unary("convert", x, "f32")
        mean = g.reduce_col("mean", xf)
        xc = xcf = g.binary("sub", xf, g.bcast_rowvec(mean, rows))   # its producer chain (the convert) lives in the first kernel
        var = g.reduce_col("mean", g.binary("mul", xcf, xcf))
        y = g.binary("mul", xcf, g.bcast_rowvec(g.unary("rsqrt", g.binary("add", var, g.const(1e-5, 1, cols))), rows))
        outs = [y, var]
        if "extra_reader" in kw:
            outs.append(g.binary("add", g.unary("abs", xcf), g.bcast_rowvec(var, rows)))
        else:
            outs.append(xc)
        g.set_outputs(outs)
        p = fs.Plan(g)
        assert p.stats()["num_launches"] == 3
        p.destroy()
        both_modes(g, [f32_to_bf16_bits((0.5 + RNG.standard_normal((rows, cols))).astype(np.float32))], f"centred bf16 input {kw}")
    g = softmax_graph(3, (1 << 19) + 8)
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 3 and p.stats()["launched_hbm_bytes"] < 4.01 * 3 * ((1 << 19) + 8) * 4
    p.destroy()
    both_modes(g, [RNG.standard_normal((3, (1 << 19) + 8)).astype(np.float32)], "softmax 3 x 512K")


def test_transposes_at_the_sizes_the_survey_times():
    # many bands of column tiles, full and ragged, over hundreds of row tiles: every element, bit for bit
    for rows, cols, dt in ((8192, 8192, "f32"), (1024, 65536 + 384, "f32"), (16384 + 64, 4096, "bf16")):
        g = Graph()
        g.set_outputs([g.transpose(g.input(rows, cols, dt))])
        p = fs.Plan(g)
        assert "in_band" in p.group_source(0)
        p.destroy()
        v = RNG.standard_normal((rows, cols)).astype(np.float32)
        x = f32_to_bf16_bits(v) if dt == "bf16" else v
        ref, out_s, _ = both_modes(g, [x], f"transpose {rows}x{cols} {dt}")
        got = out_s[0]
        np.testing.assert_array_equal(got.view(x.dtype).reshape(cols, rows), x.T)
    # bf16 tiles of large tensors are two vectors wide (512-byte rows, a 66.5 KB tile): a fused producer, rows and columns
    # that end inside a tile
    from workloads.patterns import bias_transpose
    rows, cols = 8200, 4104
    g = expose_bf16_nodes(bias_transpose(rows, cols))  # (the bf16 value also leaves as it is: its roundings are shared with the oracle)
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 1 and p.group_info(0)["elems_per_lane"] == 16 and p.group_info(0)["lds_bytes"] > 65536
    p.destroy()
    both_modes(g, [f32_to_bf16_bits(RNG.standard_normal((rows, cols)).astype(np.float32)), RNG.standard_normal((1, cols)).astype(np.float32)],
               f"bias + transpose bf16 {rows}x{cols}")


def test_column_sums_at_the_sizes_the_survey_times():
    # 4 to 16 column tiles with 16 to 64 workgroups each (fold fan-in 8 and 16), every output element
    from workloads.patterns import bias_grad, colsum
    for rows, cols, dt in ((16384, 4096, "f32"), (8192, 8192, "bf16"), (4096, 16384, "f32")):
        g = colsum(rows, cols, dt)
        p = fs.Plan(g)
        gi = p.group_info(0)
        assert p.stats()["num_launches"] == 1 and gi["lanes_per_row"] == 64 and gi["grid"] == 256
        p.destroy()
        v = (0.5 + RNG.standard_normal((rows, cols))).astype(np.float32)
        both_modes(g, [f32_to_bf16_bits(v) if dt == "bf16" else v], f"column sums {rows}x{cols} {dt}")
    g = bias_grad(16384, 4096)
    both_modes(g, [RNG.standard_normal((16384, 4096)).astype(np.float32), (0.5 + RNG.standard_normal((16384, 4096))).astype(np.float32)],
               "bias gradient 16384x4096")


def test_wide_transposes_of_bytes():
    # u8 alone is read in 16-element vectors: the tile (one float per element) is narrowed until it fits the LDS budget
    for rows, cols in ((1000, 4096), (130, 8208), (4100, 272)):
        g = Graph()
        g.set_outputs([g.transpose(g.input(rows, cols, "u8"))])
        p = fs.Plan(g)
        gi = p.group_info(0)
        assert p.stats()["num_launches"] == 1 and gi["vec_elems"] == 16 and 0 < gi["lds_bytes"] <= 65536
        p.destroy()
        v = (RNG.random((rows, cols)) < 0.3).astype(np.uint8)
        ref, out_s, _ = both_modes(g, [v], f"u8 transpose {rows}x{cols}")
        np.testing.assert_array_equal(out_s[0], v.T)


def test_transposes_inside_a_group():
    """A transpose between fused ops moves no data: consumers run in the producer's layout."""
    for rows, cols in ((130, 72), (64, 64), (512, 256), (33, 1000)):
        g = Graph()
        x = g.input(rows, cols)
        kv = g.input(cols, 1)            # per-row vector of the transposed space
        rv = g.input(1, rows)            # per-column vector of the transposed space
        y = g.unary("tanh", x)
        t = g.transpose(y)               # [cols, rows]
        u = g.binary("mul", t, g.bcast_colvec(kv, rows))
        w = g.binary("add", u, g.bcast_rowvec(rv, cols))
        rsum = g.reduce_row("sum", w)    # [cols,1]: runs down the work space's columns (grid fold)
        csum = g.reduce_col("max", w)    # [1,rows]: a row reduction of the work space
        z = g.binary("sub", w, g.bcast_rowvec(csum, cols))
        back = g.transpose(z)            # [rows, cols] again: plain store
        g.set_outputs([w, rsum, csum, z, back])
        ins = [RNG.standard_normal((rows, cols)).astype(np.float32), RNG.standard_normal((cols, 1)).astype(np.float32),
               RNG.standard_normal((1, rows)).astype(np.float32)]
        one = [0] * len(g.nodes)      # the caller's fusion plan: everything in one kernel
        p = fs.Plan(g, group_of_node=one)
        assert p.stats()["num_groups"] == 1 and p.group_info(0)["num_col_reduces"] == 1
        p.destroy()
        ref = Reference(g, ins)
        out = run_graph(g, ins, group_of_node=one)
        check_all(g, out, ref, f"in-group transposes {rows}x{cols}, one kernel")
        np.testing.assert_array_equal(out[4], out[3].T)
        both_modes(g, ins, f"in-group transposes {rows}x{cols}")   # the library's own grouping, and per-op


def test_tuning_fills_the_library_and_tuned_plans_match_the_oracle(tmp_path, monkeypatch):
    # measure-on-miss: every candidate schedule of every group is timed once and recorded; a second pass only hits
    monkeypatch.setenv("FS_PERF_LIBRARY", str(tmp_path / "perflib.tsv"))
    for cfg, rows in ((1, 300), (4, 3000), (6, 512), (5, 64)):
        g, ins, name = workload(cfg, rows)
        ref = Reference(g, ins)
        plan = fs.Plan(g)
        r = DeviceRun(plan)
        r.set_inputs(ins)
        rep = r.tune(reps=3)
        assert rep["groups"] == plan.stats()["num_groups"]
        # (groups with the same structure share their keys: the second one already hits)
        assert rep["measured"] + rep["hits"] == rep["candidates"] > rep["groups"] and rep["measured"] > rep["hits"]
        assert 0 < rep["best_usec"] <= rep["current_usec"]
        check_all(g, r.results(), ref, name + " after tuning")  # the buffers hold a normal run's results
        rep2 = r.tune(reps=3)
        assert rep2["measured"] == 0 and rep2["hits"] == rep2["candidates"] == rep["candidates"]
        plan.destroy()
        out = run_graph(g, ins)  # planned again: now with the library's schedules
        check_all(g, out, ref, name + " tuned plan")
    text = (tmp_path / "perflib.tsv").read_text()
    assert text.count("\t") >= 10 and "lanes/row" in text


def test_layered_planner_results_match_the_oracle():
    for cfg, rows in ((5, None), (6, 300), (4, 3000)):
        g, ins, name = workload(cfg, rows)
        ref = Reference(g, ins)
        out = run_graph(g, ins, mode=fs.FS_MODE_LAYERED)
        check_all(g, out, ref, name + " layered planner")


@pytest.mark.parametrize("seed,rows,ks", [(11, 33, (8, 24)), (12, 200, (36, 100)), (13, 512, (64, 128, 256)), (14, 1000, (4, 1024)),
                                          (15, 77, (130, 2)), (16, 2048, (512,))])
def test_random_dags_other_seeds_and_shapes(seed, rows, ks):
    # the benchmark's DAG generator with other seeds, row counts and column widths (ragged, tiny and wide), three planners
    g = random_dag_graph(num_nodes=120, rows=rows, ks=ks, seed=seed)
    ins = random_dag_inputs(g)
    ref = Reference(g, ins)
    for mode, label in ((fs.FS_MODE_STITCHED, "stitched"), (fs.FS_MODE_LAYERED, "layered"), (fs.FS_MODE_UNFUSED, "unfused")):
        out = run_graph(g, ins, mode=mode)
        check_all(g, out, ref, f"random dag seed {seed} rows {rows} ks {ks} {label}")


def _random_graph_case(seed, rows, cols, num_ops=40, views=False):
    """One graph of tests/graphgen.py under the three planners.  Its bf16 round trips are quantisers: they are made plan
    outputs, so the oracle can take the device's own roundings for everything downstream (see tests/parity.py)."""
    from graphgen import random_graph, random_inputs
    g = expose_bf16_nodes(random_graph(seed, rows, cols, num_ops, views=views))
    ins = random_inputs(g, seed)
    ref = Reference(g, ins)
    ill = 0
    for mode, label in ((fs.FS_MODE_STITCHED, "stitched"), (fs.FS_MODE_LAYERED, "layered"), (fs.FS_MODE_UNFUSED, "unfused")):
        out = run_graph(g, ins, mode=mode)
        # (a random graph may have a couple of outputs that are ill-conditioned throughout - differences of nearly equal values:
        # up to a quarter of all output elements may be set aside before the graph is refused as a test case)
        stats = check_all(g, out, ref, f"random graph seed {seed} {rows}x{cols} {label}", max_ill_fraction=0.25)
        ill = max(ill, sum(st["ill_conditioned"] for st in stats))
    return ill


HINTED_CASES = [  # (seed, rows, cols, views, plan arguments): looping workgroups with several tiles per trip around [1,C] values the kernel computes
    (6020, 300, 1, True, {"hint": {"lanes_per_row": 8, "wg_threads": 256, "max_workgroups": 1, "tiles_per_trip": 2}, "lds_budget_bytes": 40000, "mode": fs.FS_MODE_LAYERED}),
    (6038, 4096, 260, True, {"hint": {"lanes_per_row": 1, "wg_threads": 0, "max_workgroups": 64, "tiles_per_trip": 4}, "lds_budget_bytes": 40000, "mode": fs.FS_MODE_LAYERED}),
    (6064, 65, 63, False, {"hint": {"lanes_per_row": 1, "wg_threads": 0, "max_workgroups": 1, "tiles_per_trip": 2}}),
    (6092, 20000, 130, False, {"hint": {"lanes_per_row": 8, "wg_threads": 0, "max_workgroups": 64, "tiles_per_trip": 2}, "mode": fs.FS_MODE_LAYERED}),
    (6098, 128, 96, False, {"hint": {"lanes_per_row": 0, "wg_threads": 256, "max_workgroups": 1, "tiles_per_trip": 4}, "lds_budget_bytes": 40000, "mode": fs.FS_MODE_LAYERED}),
]


@pytest.mark.parametrize("seed,rows,cols,views,kw", HINTED_CASES)
def test_random_graphs_under_hints_that_ask_for_several_tiles_per_trip(seed, rows, cols, views, kw):
    # a [1,C] value computed inside the loop body is declared (and stored by the workgroup of row 0) under the names of a single
    # tile: such kernels take one tile per trip whatever the hint says (these five plans once produced code that did not compile)
    from graphgen import random_graph, random_inputs
    g = expose_bf16_nodes(random_graph(seed, rows, cols, 40, views=views))
    ins = random_inputs(g, seed)
    out = run_graph(g, ins, **kw)
    check_all(g, out, Reference(g, ins), f"random graph seed {seed} {rows}x{cols} {kw}", max_ill_fraction=0.25)


@pytest.mark.parametrize("seed,rows,cols", [(1, 37, 72), (2, 300, 1000), (3, 64, 64), (4, 1000, 36), (5, 5, 3000), (6, 129, 258),
                                            (7, 2048, 128), (8, 16, 4100), (9, 513, 520), (10, 70, 9000), (11, 4099, 8), (12, 260, 264)])
def test_random_graphs_with_every_op_class(seed, rows, cols):
    # ~130-node DAGs mixing all unary ops, comparisons and selects, bf16 round trips, row and column reductions of every kind,
    # transposes and both broadcasts; three planners against the oracle
    _random_graph_case(seed, rows, cols)


@pytest.mark.parametrize("seed,rows,cols", [(773, 1000, 1000), (829, 64, 16384), (868, 257, 1025)])
def test_random_graphs_whose_bf16_round_trip_hits_a_rounding_midpoint(seed, rows, cols):
    # In each of these graphs an fp32 sigmoid / tanh result equals the midpoint of two bf16 neighbours at some element.
    # The oracle rounds it to even; the device's value is one fp32 ulp lower and rounds down; a subtraction of nearly
    # equal values (773, 829) or a logarithm near 1 (868) then amplifies that one bf16 step far beyond any fixed slack.
    # With the device's roundings shared, everything downstream holds the plain fp32 tolerance.
    _random_graph_case(seed, rows, cols)


SWEEP_SHAPES = [(40, 20000), (3000, 5000), (7, 70001), (1200, 4096), (2, 2), (1, 500), (500, 1), (33000, 24), (257, 1025), (64, 16384),
                (4096, 260), (100, 33000), (65, 63), (1000, 1000), (12, 131080), (20000, 130), (3, 3), (8192, 512), (300, 300), (17, 9000)]


def test_random_graph_with_a_logarithm_next_to_one():
    # log(x) for x = 1.0019 in a tensor whose values are all ~1e-2: one fp32 ulp of x (what a 1-ulp sigmoid upstream may
    # differ by) is 1.2e-7 absolute, more than 1e-5 of the tensor's scale; the fp64 companion flags the element
    _random_graph_case(328, 257, 1025)


def test_random_graph_whose_row_sums_cancel():
    # tanh of a row sum of 5000 terms that cancel to 0.1, next to rows that sum to +-45: uncertain by ~1e-5 for any fp32
    # sum; the accumulation companion flags such rows (about 3 % here) instead of a tolerance that is loose everywhere
    assert _random_graph_case(261, 3000, 5000, 25) > 0


@pytest.mark.parametrize("first", range(int(os.environ.get("FS_SWEEP_START", "200")), int(os.environ.get("FS_SWEEP_END", "220")), 20))
def test_random_graph_sweep(first):
    # seeds 200..219 (FS_SWEEP_END widens the range: 440 is twelve times the work, ~13 minutes) over twenty shapes: tiny,
    # ragged, wide, tall, beyond one workgroup's registers; stops at the first failure
    for seed in range(first, first + 20):
        rows, cols = SWEEP_SHAPES[seed % len(SWEEP_SHAPES)]
        print(f"seed {seed} {rows}x{cols}", flush=True)
        _random_graph_case(seed, rows, cols, 25 if rows * cols > 4_000_000 else 40)


VIEW_SWEEP_SHAPES = [(65, 63), (40, 2000), (128, 96), (7, 70002), (1000, 1000), (2, 2), (300, 1), (1, 500), (4096, 260), (12, 33000), (513, 520), (64, 16384)]


@pytest.mark.parametrize("first", range(int(os.environ.get("FS_VIEW_SWEEP_START", "1000")), int(os.environ.get("FS_VIEW_SWEEP_END", "1024")), 12))
def test_random_graph_sweep_with_views_and_concats(first):
    # the same generator with the shape-modulation ops switched on: reshapes / bitcasts into another factorisation of the elements,
    # arithmetic and row reductions there, the way back, concats along columns (seams on and off vector boundaries) and rows
    for seed in range(first, first + 12):
        rows, cols = VIEW_SWEEP_SHAPES[seed % len(VIEW_SWEEP_SHAPES)]
        print(f"seed {seed} {rows}x{cols} with views", flush=True)
        _random_graph_case(seed, rows, cols, 25 if rows * cols > 2_000_000 else 35, views=True)


def test_gpu_matches_the_stored_small_cases():
    # the tiny hand-checkable cases of tests/golden/oracle_small_cases.json (written by the oracle alone), on the GPU
    import json
    import os
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.join(here, "golden"))
    import make_oracle_fixtures as mk
    stored = json.load(open(os.path.join(here, "golden", "oracle_small_cases.json")))
    for name, g, ins in mk.cases():
        ref = []
        for o, hexes, shape in zip(g.outputs, stored[name]["outputs_hex"], stored[name]["output_shapes"]):
            v = np.array([int(h, 16) for h in hexes], dtype=np.uint32).view(np.float32).reshape(shape)
            ref.append(f32_to_bf16_bits(v) if g.nodes[o].dtype == "bf16" else v)
        for mode in (fs.FS_MODE_STITCHED, fs.FS_MODE_UNFUSED):
            check_all(g, run_graph(g, ins, mode=mode), ref, f"stored case {name} mode {mode}")


def test_kernels_fused_through_a_reshape():
    # an elementwise region next to a view takes the shape of the other side and shares its kernel (Table 1: the Row schedule
    # passes through a Reshape): the region's tensors are then addressed as flat element sequences of the kernel's work space
    g = Graph()
    x, y = g.input(128, 256), g.input(128, 256)
    a = g.binary("mul", g.unary("tanh", x), y)
    r = g.reshape(a, 512, 64)
    s = g.reduce_row("sum", r)
    g.set_outputs([g.binary("sub", r, g.bcast_colvec(s, 64))])
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 1
    p.destroy()
    both_modes(g, [RNG.standard_normal((128, 256)).astype(np.float32), (1.0 + RNG.random((128, 256))).astype(np.float32)], "activation | reshape | row reduction")
    # softmax over the old rows, then a residual add and GeLU under the new shape; ragged sizes, a bf16 residual
    for rows, cols, r2, c2 in ((96, 200, 300, 64), (77, 130, 10010, 1), (4096, 260, 8192, 130)):
        g = Graph()
        x, res = g.input(rows, cols), g.input(r2, c2, "bf16")
        e = g.unary("exp", g.binary("sub", x, g.bcast_colvec(g.reduce_row("max", x), cols)))
        sm = g.binary("div", e, g.bcast_colvec(g.reduce_row("sum", e), cols))
        v = g.reshape(sm, r2, c2, op="bitcast")
        g.set_outputs([g.unary("gelu_tanh", g.binary("add", v, g.unary("convert", res, "f32")))])
        p = fs.Plan(g)
        assert p.stats()["num_launches"] == 1 and p.workspace_bytes() == 0
        p.destroy()
        both_modes(g, [RNG.standard_normal((rows, cols)).astype(np.float32), f32_to_bf16_bits(RNG.standard_normal((r2, c2)).astype(np.float32))],
                   f"softmax | bitcast | residual + gelu {rows}x{cols} -> {r2}x{c2}")
    # two views around a region, outputs on both sides of them, a predicate inside the region
    g = Graph()
    x, y = g.input(64, 96), g.input(48, 128)
    a = g.unary("sigmoid", x)
    v = g.reshape(a, 48, 128)
    b = g.binary("add", v, y)
    pred = g.cmp("gt", v, y)
    c = g.select(pred, b, g.unary("neg", y))
    g.set_outputs([g.reshape(g.unary("neg", c), 64, 96), pred, b])
    both_modes(g, [RNG.standard_normal((64, 96)).astype(np.float32), RNG.standard_normal((48, 128)).astype(np.float32)], "region between two views")


# ------------------------------------------------------------------ reshape / bitcast / concat
def test_views_of_nd_tensors_and_concats():
    """Reshape / Bitcast as zero-cost views between kernels and at the plan's edges; Concat read as one row."""
    # per-head softmax of [b, s, h, s] through views, back to the caller's 2-D shape (one kernel, no copy)
    b, h, s = 3, 5, 72
    g = Graph()
    x = g.input(b * s, h * s)
    bias = g.input(1, s)
    v = g.view_nd(x, (b, s, h, s), 3)
    z = g.binary("add", v, g.bcast_rowvec(bias, b * s * h))
    e = g.unary("exp", g.binary("sub", z, g.bcast_colvec(g.reduce_row("max", z), s)))
    y = g.binary("div", e, g.bcast_colvec(g.reduce_row("sum", e), s))
    g.set_outputs([g.reshape(y, b * s, h * s, op="bitcast")])
    ins = [RNG.standard_normal((b * s, h * s)).astype(np.float32), RNG.standard_normal((1, s)).astype(np.float32)]
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 1
    p.destroy()
    ref, out_s, _ = both_modes(g, ins, "per-head softmax through views")
    assert out_s[0].shape == (b * s, h * s)
    # a reshape between two computations: producer | consumer over the same bytes; a [1,R] vector viewed as [R,1] and
    # broadcast along rows; the reshaped intermediate is also a plan output (the producer writes it into the caller's buffer)
    g = Graph()
    x = g.input(130, 264)
    w = g.input(1, 520)
    a = g.unary("tanh", x)
    r = g.reshape(a, 520, 66)
    wcol = g.reshape(w, 520, 1)
    t = g.binary("mul", r, g.bcast_colvec(wcol, 66))
    sm = g.reduce_row("sum", t)
    back = g.reshape(g.binary("sub", t, g.bcast_colvec(sm, 66)), 130, 264)
    g.set_outputs([back, r, g.reshape(sm, 1, 520)])
    ins = [RNG.standard_normal((130, 264)).astype(np.float32), RNG.standard_normal((1, 520)).astype(np.float32)]
    ref, out_s, out_u = both_modes(g, ins, "reshape between kernels")
    # bf16 payload through a view; a chain of views
    g = Graph()
    x = g.input(64, 96, "bf16")
    v2 = g.reshape(g.reshape(g.reshape(x, 96, 64), 1, 6144, op="bitcast"), 32, 192)
    g.set_outputs([g.unary("neg", v2), g.reduce_row("max", g.unary("convert", v2, "f32"))])
    both_modes(g, [f32_to_bf16_bits(RNG.standard_normal((64, 96)).astype(np.float32))], "chain of views, bf16")
    # concat along columns feeding a normalisation (ragged tail, a seam that is not a multiple of the widest vector),
    # along rows feeding column and row reductions, of bf16 tensors, and as a plan output of its own (a copy kernel)
    for rows, c0, c1 in ((300, 96, 160), (77, 30, 34), (1000, 8, 1000), (5, 4100, 12)):
        g = Graph()
        ia, ib = g.input(rows, c0), g.input(rows, c1)
        c = g.concat(ia, ib)
        m = g.reduce_row("mean", c)
        g.set_outputs([g.binary("sub", c, g.bcast_colvec(m, c0 + c1)), c])
        ins = [RNG.standard_normal((rows, c0)).astype(np.float32), RNG.standard_normal((rows, c1)).astype(np.float32)]
        ref, out_s, _ = both_modes(g, ins, f"concat cols {rows}x({c0}+{c1})")
        np.testing.assert_array_equal(out_s[1], np.concatenate(ins, axis=1))
    for r0, r1, cols, dt in ((100, 28, 64, "f32"), (1, 700, 130, "f32"), (513, 511, 256, "bf16")):
        g = Graph()
        ia, ib = g.input(r0, cols, dt), g.input(r1, cols, dt)
        c = g.concat(ia, ib, "rows")
        cf = g.unary("convert", c, "f32") if dt != "f32" else c
        g.set_outputs([g.reduce_col("sum", cf), g.reduce_row("max", g.unary("abs", cf)), c])
        ins = [RNG.standard_normal((r0, cols)).astype(np.float32), RNG.standard_normal((r1, cols)).astype(np.float32)]
        if dt == "bf16":
            ins = [f32_to_bf16_bits(a) for a in ins]
        ref, out_s, _ = both_modes(g, ins, f"concat rows ({r0}+{r1})x{cols} {dt}")
        np.testing.assert_array_equal(out_s[2], np.concatenate(ins, axis=0))
    # an operand computed by the graph (materialised first), and a concat of a view
    g = Graph()
    ia, ib = g.input(64, 48), g.input(32, 96)
    c = g.concat(g.unary("tanh", ia), g.reshape(ib, 64, 48))
    g.set_outputs([g.reduce_row("sum", c), g.unary("sigmoid", c)])
    both_modes(g, [RNG.standard_normal((64, 48)).astype(np.float32), RNG.standard_normal((32, 96)).astype(np.float32)], "concat of computed + view")
