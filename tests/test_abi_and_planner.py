"""Host-side tests of the C-ABI library: symbols, validation errors, grouping, schedules, LDS plan.

No GPU is needed: fs_plan_create is host-only (kernels are compiled for gfx950 by the run-time
compiler, not loaded).  Compute entry points are not called here.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1811_05213_amd as fs
from paper_1811_05213_amd import binding
from workloads import (Graph, elementwise20_graph, layernorm_gelu_graph, min_hbm_bytes, multi_reduce_graph,
                       random_dag_graph, softmax_graph)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def built_lib():
    if not os.path.exists(fs.LIB_PATH):
        from paper_1811_05213_amd import build
        build.build()
    return fs.lib()


def test_library_exports_every_declared_symbol(built_lib):
    text = open(os.path.join(ROOT, "include", "fs.h")).read()
    declared = set(re.findall(r"\b(fs_[a-z_0-9]+)\s*\(", text))
    declared -= {"fs_plan"}  # the opaque type
    assert {"fs_plan_create", "fs_plan_run", "fs_plan_destroy", "fs_plan_workspace_bytes", "fs_last_error"} <= declared
    raw = ctypes.CDLL(fs.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(raw, name), f"libfs.so does not export {name}"


def _status(graph, **kw):
    try:
        fs.Plan(graph, **kw).destroy()
        return "FS_OK"
    except fs.FsError as e:
        return e.status_name


def test_validation_errors():
    # operand id not smaller than node id (dangling / cycle)
    g = Graph()
    x = g.input(4, 8)
    y = g.unary("neg", x)
    g.nodes[y].ins = (5,)
    g.set_outputs([y])
    assert _status(g) == "FS_ERR_BAD_GRAPH"
    # arity
    g = Graph()
    x = g.input(4, 8)
    y = g.binary("add", x, x)
    g.nodes[y].ins = (x,)
    g.set_outputs([y])
    assert _status(g) == "FS_ERR_BAD_GRAPH"
    # shape mismatch
    g = Graph()
    a, b = g.input(4, 8), g.input(4, 9)
    y = g.binary("add", a, b)
    g.set_outputs([y])
    assert _status(g) == "FS_ERR_SHAPE"
    g = Graph()
    a = g.input(4, 8)
    r = g.reduce_row("sum", a)
    g.nodes[r].cols = 2
    g.set_outputs([r])
    assert _status(g) == "FS_ERR_SHAPE"
    # dtype rules
    g = Graph()
    a, b = g.input(4, 8), g.input(4, 8)
    c = g.cmp("gt", a, b)
    g.nodes[c].dtype = "f32"
    g.set_outputs([c])
    assert _status(g) == "FS_ERR_DTYPE"
    g = Graph()
    a, b = g.input(4, 8), g.input(4, 8)
    s = g.select(a, a, b)  # predicate is not u8
    g.set_outputs([s])
    assert _status(g) == "FS_ERR_DTYPE"
    # outputs: a broadcast is never materialised; duplicates; out of range
    g = Graph()
    v = g.input(1, 8)
    b = g.bcast_rowvec(v, 4)
    g.set_outputs([b])
    assert _status(g) == "FS_ERR_BAD_GRAPH"
    g = softmax_graph(8, 64)
    g.set_outputs(g.outputs * 2)
    assert _status(g) == "FS_ERR_BAD_GRAPH"
    g = softmax_graph(8, 64)
    g.set_outputs([999])
    assert _status(g) == "FS_ERR_BAD_GRAPH"


def test_degenerate_graphs_are_refused():
    # empty tensors, no outputs, an input as an output: distinct statuses, nothing planned
    for r, c in ((0, 8), (8, 0), (-1, 4)):
        g = Graph()
        x = g.input(4, 8)
        y = g.unary("neg", x)
        g.set_outputs([y])
        for n in (x, y):
            g.nodes[n].rows, g.nodes[n].cols = r, c
        assert _status(g) == "FS_ERR_SHAPE"
    g = Graph()
    g.input(4, 8)
    g.set_outputs([])
    assert _status(g) == "FS_ERR_INVALID_ARG"
    g = Graph()
    x = g.input(4, 8)
    g.set_outputs([x])
    assert _status(g) == "FS_ERR_BAD_GRAPH"


def test_invalid_arguments(built_lib):
    desc = binding.fs_graph_desc()
    h = ctypes.c_void_p()
    assert built_lib.fs_plan_create(None, ctypes.byref(h)) == 1
    assert b"NULL" in built_lib.fs_last_error()
    desc.abi_version = 77
    assert built_lib.fs_plan_create(ctypes.byref(desc), ctypes.byref(h)) == 1
    assert built_lib.fs_plan_destroy(None) == 0
    n = ctypes.c_size_t()
    assert built_lib.fs_plan_workspace_bytes(None, ctypes.byref(n)) == 1


@pytest.mark.parametrize("name,graph,nodes", [
    ("softmax", softmax_graph(256, 1024), 5),
    ("layernorm", layernorm_gelu_graph(16384, 1024), 13),
    ("elementwise20", elementwise20_graph(65536, 1024), 20),
    ("multi_reduce", multi_reduce_graph(65536, 512), 5),
])
def test_workloads_1_to_4_are_one_stitched_kernel(name, graph, nodes):
    p = fs.Plan(graph)
    st = p.stats()
    assert st["num_groups"] == 1 and st["num_launches"] == 1
    assert st["min_hbm_bytes"] == min_hbm_bytes(graph) == st["launched_hbm_bytes"]
    gi = p.group_info(0)
    assert gi["num_nodes"] == nodes
    assert gi["dom_rows"] == graph.nodes[0].rows and gi["dom_cols"] == graph.nodes[0].cols
    # Section 4.4: thread block size is a multiple of the wavefront size, at most 1024
    assert gi["wg_threads"] % 64 == 0 and 64 <= gi["wg_threads"] <= 1024
    assert gi["lanes_per_row"] & (gi["lanes_per_row"] - 1) == 0
    assert gi["wg_threads"] == gi["rows_per_iter"] * gi["lanes_per_row"]
    assert gi["grid"] >= 1 and gi["lds_bytes"] <= 65536
    # 128-bit accesses for the widest dtype
    assert gi["vec_elems"] == (8 if name == "layernorm" else 4)
    src = p.group_source(0)
    assert p.group_kernel_name(0) in src and "__launch_bounds__" in src
    # the unfused executor: one launch per compute node, more traffic
    u = fs.Plan(graph, mode=fs.FS_MODE_UNFUSED)
    su = u.stats()
    assert su["num_launches"] == nodes and su["launched_hbm_bytes"] > st["launched_hbm_bytes"]
    assert u.workspace_bytes() > 0
    p.destroy()
    u.destroy()


def test_softmax_reductions_share_lds_slots():
    # Section 5.1.3: Reduce.2 reuses the buffer of Reduce.1.  With a row spread over 4 wavefronts the
    # two row reductions together use one ping-pong pair of 4-float slots, not one buffer each.
    p = fs.Plan(softmax_graph(256, 1024), hint={"lanes_per_row": 256, "wg_threads": 256})
    gi = p.group_info(0)
    assert gi["num_row_reduces"] == 2
    assert gi["lds_bytes"] == 2 * 1 * 4 * 1 * 4  # 2 halves x 1 row-group x 4 waves x 1 reduction x 4 B
    p.destroy()
    # a row inside one wavefront needs no LDS at all
    p = fs.Plan(softmax_graph(65536, 1024))
    assert p.group_info(0)["lanes_per_row"] == 64 and p.group_info(0)["lds_bytes"] == 0
    p.destroy()


def test_single_block_schedule_is_always_valid():
    # Section 4.3: split_dim = 0, sword = 1 (one thread block) is valid for every fused computation
    for g in (softmax_graph(300, 1000), layernorm_gelu_graph(77, 1024), multi_reduce_graph(1000, 512), elementwise20_graph(64, 1024)):
        p = fs.Plan(g, hint={"max_workgroups": 1})
        assert p.stats()["num_groups"] == 1 and p.group_info(0)["grid"] == 1
        p.destroy()


def test_lds_budget():
    g = multi_reduce_graph(4096, 512)
    # caller-given single group that cannot fit: distinct status, no abort
    grp = [0] * len(g.nodes)
    assert _status(g, group_of_node=grp, lds_budget_bytes=256) == "FS_ERR_LDS_BUDGET"
    assert _status(g, group_of_node=grp) == "FS_OK"
    # greedy grouping under the same budget cannot place the column reductions either
    assert _status(g, lds_budget_bytes=256) == "FS_ERR_LDS_BUDGET"
    # but row-only work still plans: the budget only removes what needs LDS
    assert _status(softmax_graph(64, 1024), lds_budget_bytes=256) == "FS_OK"


def test_caller_grouping_checked():
    g = softmax_graph(64, 256)
    ids = g.compute_ids()
    ok = [0] * len(g.nodes)
    assert _status(g, group_of_node=ok) == "FS_OK"
    # m | d,e | s | y : legal chain of four groups
    grp = [0] * len(g.nodes)
    for k, i in enumerate(ids):
        grp[i] = [0, 1, 1, 2, 3][k]
    p = fs.Plan(g, group_of_node=grp)
    assert p.stats()["num_groups"] == 4
    p.destroy()
    # y with m but without d,e,s: group {m,y} both feeds and consumes group {d,e,s} -> cycle
    grp = [0] * len(g.nodes)
    for k, i in enumerate(ids):
        grp[i] = [0, 1, 1, 1, 0][k]
    assert _status(g, group_of_node=grp) == "FS_ERR_UNSUPPORTED"
    # a column reduction result cannot be consumed inside its own group
    g = Graph()
    x = g.input(64, 32)
    c = g.reduce_col("sum", x)
    y = g.binary("sub", x, g.bcast_rowvec(c, 64))
    g.set_outputs([y])
    assert _status(g, group_of_node=[0] * len(g.nodes)) == "FS_ERR_UNSUPPORTED"
    p = fs.Plan(g)  # the greedy grouper cuts there instead
    assert p.stats()["num_groups"] == 2
    p.destroy()


def _check_grouping(g, p):
    """SchdConsistent conditions (Section 3.2) as properties of the result."""
    grp = p.node_groups()
    ngroups = p.stats()["num_groups"]
    free = {"input", "const", "bcast_rowvec", "bcast_colvec"}
    users = {i: [] for i in range(len(g.nodes))}
    for i, n in enumerate(g.nodes):
        for o in n.ins:
            users[o].append(i)

    def real_users(i):
        out = []
        for u in users[i]:
            out += real_users(u) if g.nodes[u].op in ("bcast_rowvec", "bcast_colvec") else [u]
        return out

    def source(o):
        return g.nodes[o].ins[0] if g.nodes[o].op in ("bcast_rowvec", "bcast_colvec") else o

    for i, n in enumerate(g.nodes):
        if n.op in free:
            assert grp[i] == -1
            continue
        assert 0 <= grp[i] < ngroups
        # launch order is a topological order of the groups: producers never come later
        for o in n.ins:
            s = source(o)
            if g.nodes[s].op not in free:
                assert grp[s] <= grp[i], f"node {i} in group {grp[i]} reads node {s} of later group {grp[s]}"
    return grp


def test_random_dag_grouping_properties():
    g = random_dag_graph()
    p = fs.Plan(g)
    st = p.stats()
    grp = _check_grouping(g, p)
    assert st["num_groups"] < 40, "200 nodes should fuse into far fewer launches"
    assert st["launched_hbm_bytes"] >= st["min_hbm_bytes"]
    u = fs.Plan(g, mode=fs.FS_MODE_UNFUSED)
    assert u.stats()["num_launches"] == len(g.compute_ids()) == 200
    assert u.stats()["launched_hbm_bytes"] > st["launched_hbm_bytes"]
    # a column-direction reduction result only exists after the whole grid has run: its consumers are in later groups
    gi = {k: p.group_info(k) for k in range(st["num_groups"])}
    assert st["num_groups"] <= 8
    p.destroy()
    u.destroy()


def test_dead_nodes_are_not_executed():
    g = Graph()
    x = g.input(16, 64)
    y = g.unary("tanh", x)
    g.unary("exp", x)  # dead
    g.set_outputs([y])
    p = fs.Plan(g)
    assert p.stats()["num_groups"] == 1 and p.group_info(0)["num_nodes"] == 1
    assert p.node_groups()[2] == -1
    p.destroy()


def test_ragged_and_degenerate_shapes_plan():
    for rows, cols in ((1, 1), (1, 777), (300, 1), (37, 1000), (5, 3), (3, 20000)):
        g = softmax_graph(rows, cols)
        p = fs.Plan(g)
        gi = p.group_info(0)
        assert gi["elems_per_lane"] * gi["lanes_per_row"] >= cols
        p.destroy()
    # rows too long for one workgroup's registers are walked in chunks (one row per workgroup, recomputation per stage)
    p = fs.Plan(softmax_graph(40, 1 << 20))
    gi = p.group_info(0)
    assert p.stats()["num_launches"] == 1 and gi["elems_per_lane"] * gi["lanes_per_row"] < (1 << 20) and gi["rows_per_iter"] == 1
    src = p.group_source(0)
    assert src.count("const int vbase = RESV + ch * (NVL * L);") == 3  # max pass, sum pass, output pass
    p.destroy()
    # between 32768 and 65536 columns a softmax row still fits the registers (64 elements per lane); LayerNorm+GeLU with its
    # three per-column vectors would spill hundreds of bytes there, which plan creation detects from the compiled kernel: the
    # row is walked in chunks instead (with or without a resident part)
    p = fs.Plan(softmax_graph(4, 65536))
    assert p.group_info(0)["elems_per_lane"] == 64 and "ch" not in re.findall(r"for \(int (\w+) = ", p.group_source(0))
    p.destroy()
    p = fs.Plan(layernorm_gelu_graph(4, 65536))
    assert p.group_info(0)["elems_per_lane"] <= 32 and "ch" in re.findall(r"for \(int (\w+) = ", p.group_source(0))
    p.destroy()
    # column reductions over wide rows run by column tiles
    gw = Graph()
    xw = gw.input(100, 50000)
    gw.set_outputs([gw.reduce_col("sum", xw)])
    p = fs.Plan(gw)
    gi = p.group_info(0)
    assert gi["grid"] % -(-50000 // (gi["elems_per_lane"] * gi["lanes_per_row"])) == 0 and "tile * CW" in p.group_source(0)
    p.destroy()
    # ... but not together with a column reduction in the same kernel: refused cleanly
    g = multi_reduce_graph(4, 1 << 17)
    assert _status(g, group_of_node=[0 if n.op not in ("input", "const", "bcast_rowvec", "bcast_colvec") else -1 for n in g.nodes]) \
        == "FS_ERR_UNSUPPORTED"


def _lds_plan(graph, **kw):
    p = fs.Plan(graph, **kw)
    try:
        lines = [ln.strip() for ln in p.group_source(0).splitlines() if "LDS plan:" in ln]
        assert len(lines) == 1, lines
        return lines[0], p.group_info(0), p.group_source(0)
    finally:
        p.destroy()


def _layernorm_f32(rows, cols):
    g = Graph()
    x, gam, bet = g.input(rows, cols), g.input(1, cols), g.input(1, cols)
    xc = g.binary("sub", x, g.bcast_colvec(g.reduce_row("mean", x), cols))
    rstd = g.unary("rsqrt", g.binary("add", g.reduce_row("mean", g.binary("mul", xc, xc)), g.const(1e-5, rows, 1)))
    g.set_outputs([g.binary("add", g.binary("mul", g.binary("mul", xc, g.bcast_colvec(rstd, cols)), g.bcast_rowvec(gam, rows)), g.bcast_rowvec(bet, rows))])
    return g


def test_shared_memory_planning_for_rows_walked_in_chunks():
    # Section 5.1 for kernels that walk a row once per stage: what several passes need may keep (the head of) the row in LDS.
    from workloads.patterns import masked_softmax
    # space sharing (5.1.3): exp(x - max) has users in two passes (the row sum, the division), dominates x seen from the root and
    # has x's element size: it takes over x's slot, and the last pass reads it back instead of computing exp again
    plan, gi, src = _lds_plan(softmax_graph(2048, 100000))
    assert re.search(r"slot 0 \(4 B/element\): v\d+ input, then v\d+ exp \(dominates it\)$", plan), plan
    assert "slot 1" not in plan and "recomputed instead" not in plan
    last_pass = src[src.rindex("for (int ch = 0; ch < CT; ++ch)"):]
    buffered, recomputed = last_pass.split("} else {")
    assert "fs_exp" not in buffered and "fs_load_row_chunk_lds" in buffered and "fs_exp" in recomputed  # (chunks beyond the LDS head: as without the buffer)
    # x - max has one user (exp): not a candidate
    assert " sub" not in plan
    # LayerNorm on fp32 rows: x - mean (users: the variance pass, the last pass) overwrites x
    plan, gi, src = _lds_plan(_layernorm_f32(512, 40000))
    assert re.search(r"slot 0 \(4 B/element\): v\d+ input, then v\d+ sub \(dominates it\)$", plan), plan
    # ... on bf16 rows it cannot (an fp32 result does not fit a bf16 slot lane by lane) and a slot of its own (4 B/element) beside
    # the row exceeds the LDS: given up, i.e. recomputed by each pass (size shrinking, 5.1.2), while the input keeps the whole row
    plan, gi, src = _lds_plan(layernorm_gelu_graph(4096, 65536))
    assert plan.startswith("// LDS plan: 4 of 4 chunks per row; slot 0 (2 B/element): v0 input")
    assert re.search(r"recomputed instead: v\d+ sub \(inexpensive", plan) and gi["lds_bytes"] >= 131072
    # the order in which buffers are given up: results of inexpensive ops before those of expensive ones
    plan, gi, src = _lds_plan(masked_softmax(512, 70000))
    assert plan.index("add (inexpensive") < plan.index("exp (expensive") and "slot 1 (2 B/element)" in plan
    # an input that is only read on the way to a buffered result needs no slot of its own: on fp32 rows x * scale + mask takes over
    # x's slot in the first pass, and the mask is never read again
    plan, gi, src = _lds_plan(masked_softmax(512, 70000, "f32"))
    assert re.search(r"slot 0 \(4 B/element\): v\d+ input, then v\d+ add \(dominates it\), then v\d+ exp \(dominates it\)$", plan), plan
    # a caller's LDS budget bounds the buffers: only the head of the row is kept
    plan, gi, src = _lds_plan(softmax_graph(2048, 100000), lds_budget_bytes=70000)
    assert plan.startswith("// LDS plan: 1 of 4 chunks per row") and gi["lds_bytes"] <= 70000


def test_performance_library_drives_the_schedule(tmp_path, monkeypatch):
    # schedule tuning = enumerate the candidates, look each kernel up in the library, keep the fastest recorded one
    lib_file = tmp_path / "perflib.tsv"
    monkeypatch.setenv("FS_PERF_LIBRARY", str(lib_file))
    g = softmax_graph(300, 1000)
    p0 = fs.Plan(g)
    base = p0.group_info(0)
    k0 = p0.group_perf_key(0)
    assert k0.startswith(p0.group_kernel_name(0) + ":R300:")
    hinted = fs.Plan(g, hint={"lanes_per_row": base["lanes_per_row"] * 2, "wg_threads": base["wg_threads"]})
    k1 = hinted.group_perf_key(0)
    assert k1 != k0 and hinted.group_info(0)["lanes_per_row"] == 2 * base["lanes_per_row"]

    # only the candidate is recorded: an unmeasured base schedule is not displaced
    lib_file.write_text(f"# test library\n{k1}\t5.0\n")
    p = fs.Plan(g)
    assert p.group_perf_key(0) == k0
    p.destroy()
    # both recorded, the candidate faster: it is chosen ...
    lib_file.write_text(f"{k0}\t10.0\n{k1}\t5.0\n")
    p = fs.Plan(g)
    assert p.group_perf_key(0) == k1 and p.group_info(0)["lanes_per_row"] == 2 * base["lanes_per_row"]
    p.destroy()
    # ... unless the caller opts out, or passes a hint of its own
    p = fs.Plan(g, mode=fs.FS_MODE_NO_PERFLIB)
    assert p.group_perf_key(0) == k0
    p.destroy()
    p = fs.Plan(g, hint={"wg_threads": base["wg_threads"]})
    assert p.group_info(0)["lanes_per_row"] == base["lanes_per_row"]
    p.destroy()
    # a candidate inside the measurement noise (5 %) does not displace the analytic schedule
    lib_file.write_text(f"{k0}\t10.0\n{k1}\t9.6\n")
    p = fs.Plan(g)
    assert p.group_perf_key(0) == k0
    p.destroy()
    # a later record overrides an earlier one; malformed lines are skipped
    with open(lib_file, "a") as f:
        f.write(f"garbage line\n{k1}\t5.0\n{k1}\t50.0\n")
    p = fs.Plan(g)
    assert p.group_perf_key(0) == k0
    p.destroy()
    p0.destroy()
    hinted.destroy()


def test_huge_row_counts_stay_inside_the_launch_limits():
    # one workgroup per row tile until a launch would hold 2^31 lanes; then the workgroups loop over tiles
    g = Graph()
    x = g.input(1 << 28, 4)
    g.set_outputs([g.unary("exp", x)])
    p = fs.Plan(g)
    gi = p.group_info(0)
    tiles = -(-(1 << 28) // gi["rows_per_iter"])
    assert gi["grid"] * gi["wg_threads"] < 2 ** 31 and gi["grid"] <= tiles
    p.destroy()


def test_spill_feedback_relieves_register_pressure():
    # plan creation reads every kernel's scratch size from the compiled code object; a kernel that spills hundreds of bytes is
    # planned again with a milder row form or half the workgroup.  LayerNorm + GeLU over 65536 bf16 columns would hold 64
    # elements per lane plus three per-column operands (~800 bytes of scratch): it ends up walking the row in chunks instead
    p = fs.Plan(layernorm_gelu_graph(4, 65536))
    assert p.group_info(0)["elems_per_lane"] <= 32 and "int ch =" in p.group_source(0)
    p.destroy()
    # the same row without the operands fits: softmax keeps all 64 elements per lane in registers
    p = fs.Plan(softmax_graph(4, 65536))
    assert p.group_info(0)["elems_per_lane"] == 64 and "int ch =" not in p.group_source(0)
    p.destroy()
    # LayerNorm backward over 8192 columns stays one kernel (a handful of spilled registers, under 128 bytes, is tolerated)
    from workloads import layernorm_grad_graph
    p = fs.Plan(layernorm_grad_graph(4096, 8192))
    assert p.stats()["num_launches"] == 1 and p.group_info(0)["wg_threads"] in (512, 1024)
    p.destroy()


def test_occupancy_feedback_for_1024_lane_workgroups():
    # two 1024-lane workgroups share a CU only at <= 64 vector registers; a kernel a few registers above that is compiled again
    # with the compiler asked for 8 wavefronts per SIMD, and keeps that form only if nothing spills
    p = fs.Plan(softmax_graph(2048, 32768))
    assert p.group_info(0)["wg_threads"] == 1024 and p.group_info(0)["elems_per_lane"] == 32
    src = p.group_source(0)
    if "amdgpu_waves_per_eu(8)" in src:  # taken: the compiled kernel must be spill-free (the plan would have gone back otherwise)
        assert p.stats()["num_launches"] == 1
    p.destroy()
    # kernels that are not 1024 lanes wide, or fit anyway, carry no such request
    for g in (softmax_graph(4096, 4096), softmax_graph(4096, 16384)):
        p = fs.Plan(g)
        assert "amdgpu_waves_per_eu" not in p.group_source(0)
        p.destroy()


def test_work_span_and_layered_planner():
    # Work/Span: roots have span 0, everything else 1 + the largest span of its users; a layer has no internal dependences
    g = random_dag_graph()
    p = fs.Plan(g, mode=fs.FS_MODE_LAYERED)
    span = p.node_spans()
    free = ("input", "const", "bcast_rowvec", "bcast_colvec")
    users = {i: [] for i in range(len(g.nodes))}

    def real_users(i):
        out = []
        for u in users[i]:
            out += real_users(u) if g.nodes[u].op in free else [u]
        return out
    for i, n in enumerate(g.nodes):
        for o in n.ins:
            users[o].append(i)
    live = [s >= 0 for s in span]
    for i, n in enumerate(g.nodes):
        if n.op in free:
            assert span[i] == -1
            continue
        if not live[i]:
            continue
        us = [u for u in real_users(i) if live[u]]
        assert span[i] == (1 + max(span[u] for u in us) if us else 0)
        for o in n.ins:
            assert g.nodes[o].op in free or span[o] > span[i]
    assert all(span[o] >= 0 for o in g.outputs) and min(span[o] for o in g.outputs) == 0
    # the layered plan is a valid plan: every live compute node in exactly one group, launch order respects dependences
    grp = p.node_groups()
    for i, n in enumerate(g.nodes):
        if n.op not in free and live[i]:
            assert grp[i] >= 0
            for o in n.ins:
                src = o
                while g.nodes[src].op in ("bcast_rowvec", "bcast_colvec"):
                    src = g.nodes[src].ins[0]
                if g.nodes[src].op not in free:
                    assert grp[src] <= grp[i]
    d = fs.Plan(g)
    # the default planner (exact cycle test, any user's group, sibling merging across layers) needs far fewer launches
    assert d.stats()["num_launches"] < p.stats()["num_launches"] <= len(g.compute_ids())
    assert d.node_spans() == span
    p.destroy()
    d.destroy()
    # on the chain-like workloads both planners find the single kernel
    for g2 in (softmax_graph(300, 1000), layernorm_gelu_graph(77, 1024), elementwise20_graph(64, 1024)):
        p = fs.Plan(g2, mode=fs.FS_MODE_LAYERED)
        assert p.stats()["num_launches"] == 1
        p.destroy()


def test_few_long_rows_are_split_over_workgroups():
    # [R,1]-only results over a handful of very long rows: one workgroup per row segment, about 512 in all, a per-row fold
    def norms(rows, cols, keep_full=False):
        g = Graph()
        x = g.input(rows, cols)
        outs = [g.unary("sqrt", g.reduce_row("sum", g.binary("mul", x, x))), g.reduce_row("max", x)]
        if keep_full == "before":
            outs.append(g.unary("neg", x))
        if keep_full == "after":
            outs.append(g.binary("div", x, g.bcast_colvec(outs[0], cols)))
        g.set_outputs(outs)
        return g
    p = fs.Plan(norms(4, 1 << 22))
    gi = p.group_info(0)
    assert p.stats()["num_launches"] == 1 and gi["grid"] == 512 and gi["wg_threads"] == 256 and gi["scratch_bytes"] > 0
    assert "constexpr int S = 128" in p.group_source(0)
    assert fs.Plan(norms(4, 1 << 22), hint={"max_workgroups": 64}).group_info(0)["grid"] == 64
    # an [R,C] output computed before any reduction result is stored by the segment workgroups
    p = fs.Plan(norms(4, 1 << 22, keep_full="before"))
    assert p.stats()["num_launches"] == 1 and p.group_info(0)["grid"] == 512 and "fs_store_row" in p.group_source(0)
    # one that depends on a reduction, many rows, or rows a workgroup holds in registers: the ordinary forms
    p = fs.Plan(norms(40, 1 << 20, keep_full="after"))
    assert p.stats()["num_launches"] == 1 and p.group_info(0)["grid"] == 40
    assert fs.Plan(norms(4096, 1 << 18)).group_info(0)["grid"] == 4096
    assert fs.Plan(norms(4, 1 << 14)).group_info(0)["grid"] == 4
    # up to 32 such rows, groups that cannot take this form are not formed: a softmax becomes max | sum of the exponentials |
    # exponentials again and divide, three launches that each fill the device instead of one on 2 CUs; the exponentials are
    # computed by both kernels that need them rather than stored by one and read by the other (x is read three times and
    # the result written once: four passes, not five)
    g = softmax_graph(2, 1 << 20)
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 3 and [p.group_info(i)["grid"] for i in range(2)] == [256, 256]
    assert "fs_store_row" not in p.group_source(1) and "constexpr int S = 128" in p.group_source(1) and "fs_exp" in p.group_source(1)
    assert "fs_exp" in p.group_source(2) and p.group_info(2)["num_nodes"] == 3
    assert p.stats()["launched_hbm_bytes"] == 2 * min_hbm_bytes(g) + 5 * (2 * 4)  # + the [R,1] maxima (written once, read twice) and sums (written, read)


def _batchnorm_like(rows, cols, extra_reader=False, keep_as_output=False):
    g = Graph()
    x = g.input(rows, cols)
    mean = g.reduce_col("mean", x)
    xc = g.binary("sub", x, g.bcast_rowvec(mean, rows), name="xc")
    var = g.reduce_col("mean", g.binary("mul", xc, xc))
    rstd = g.unary("rsqrt", g.binary("add", var, g.const(1e-5, 1, cols)))
    y = g.binary("mul", xc, g.bcast_rowvec(rstd, rows))
    outs = [y, var]
    if extra_reader:  # a third kernel that needs xc as well (it consumes var, so it cannot join the kernel that folds var)
        outs.append(g.binary("add", g.unary("abs", xc), g.bcast_rowvec(var, rows)))
    if keep_as_output:
        outs.append(xc)
    g.set_outputs(outs)
    return g, xc


def test_values_needed_by_two_kernels_are_computed_twice_when_that_moves_fewer_bytes():
    rows, cols = 8192, 2048
    full, vec = rows * cols * 4, cols * 4
    # column statistics force three kernels; the centred values are needed by the second (variance) and the third (result):
    # the third computes them again from x and the means instead of reading a copy the second would have to store
    g, xc = _batchnorm_like(rows, cols)
    p = fs.Plan(g)
    st = p.stats()
    assert st["num_launches"] == 3 and p.workspace_bytes() < full  # no [R,C] value passes through the workspace
    # x read three times, y written once; the means written once and read twice, the variances written and read once
    assert st["launched_hbm_bytes"] == 4 * full + 5 * vec
    assert p.node_groups()[xc] == 1 and [p.group_info(k)["num_nodes"] for k in range(3)] == [1, 3, 4]
    own = [max(k, 0) for k in p.node_groups()]
    p.destroy()
    # the caller's own plan is taken as it is: the value is stored by its kernel and read by the other
    q = fs.Plan(g, group_of_node=own)
    assert q.stats()["num_launches"] == 3 and q.stats()["launched_hbm_bytes"] == 5 * full + 4 * vec and q.workspace_bytes() > full
    q.destroy()
    # a third reader in the last kernel: still one copy there, nothing stored
    g3, _ = _batchnorm_like(rows, cols, extra_reader=True)
    p = fs.Plan(g3)
    assert p.stats()["num_launches"] == 3 and p.stats()["launched_hbm_bytes"] == 5 * full + 5 * vec and p.workspace_bytes() < full
    p.destroy()
    # a plan output exists in memory anyway: the last kernel reads it (as many bytes as reading x)
    g2, _ = _batchnorm_like(rows, cols, keep_as_output=True)
    p = fs.Plan(g2)
    assert p.stats()["launched_hbm_bytes"] == 5 * full + 4 * vec and p.workspace_bytes() < full
    p.destroy()
    # the one-launch-per-op executor is untouched
    u = fs.Plan(g, mode=fs.FS_MODE_UNFUSED)
    assert u.stats()["num_launches"] == len(g.compute_ids())
    u.destroy()


def test_hinted_plans_that_once_failed_to_compile():
    # several tiles per trip asked for (by hint) around [1,C] values that the kernel computes inside its loop body: the
    # kernel takes one tile per trip, and its code compiles (plan creation compiles every kernel, no GPU needed)
    import sys
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from graphgen import random_graph
    cases = [(6020, 300, 1, True, {"hint": {"lanes_per_row": 8, "wg_threads": 256, "max_workgroups": 1, "tiles_per_trip": 2}, "lds_budget_bytes": 40000, "mode": fs.FS_MODE_LAYERED}),
             (6064, 65, 63, False, {"hint": {"lanes_per_row": 1, "wg_threads": 0, "max_workgroups": 1, "tiles_per_trip": 2}}),
             (6098, 128, 96, False, {"hint": {"lanes_per_row": 0, "wg_threads": 256, "max_workgroups": 1, "tiles_per_trip": 4}, "lds_budget_bytes": 40000, "mode": fs.FS_MODE_LAYERED})]
    for seed, rows, cols, views, kw in cases:
        p = fs.Plan(random_graph(seed, rows, cols, 40, views=views), **kw)
        assert p.stats()["num_launches"] >= 1
        p.destroy()


def test_tile_order_of_wide_transposes_and_column_tiles_of_column_reductions():
    from workloads.patterns import colsum, transpose
    # 2-D transpose tiles are walked in bands of column tiles: 4 KB of a row per band (8 tiles of f32, 16 of bf16), twice
    # that with 32 row tiles or fewer (a bf16 tile is 256 columns wide: two vectors per lane); no bands where a row has no more tiles than a band
    for rows, cols, dt, band in ((8192, 8192, "f32", 8), (1024, 65536, "f32", 16), (16384, 4096, "bf16", 8), (65536, 1024, "f32", 0)):
        p = fs.Plan(transpose(rows, cols, dt))
        src = p.group_source(0)
        assert (f"TCB = {band}," in src) if band else ("in_band" not in src), (rows, cols, dt)
        p.destroy()
    # column reductions without row reductions: tiles of 64 lanes x 64 bytes from 513 f32 columns on, one fold per tile
    for rows, cols, dt, elems, tiles in ((16384, 4096, "f32", 16, 4), (8192, 8192, "bf16", 32, 4), (65536, 1024, "f32", 16, 1), (65536, 512, "f32", 8, 1)):
        p = fs.Plan(colsum(rows, cols, dt))
        gi = p.group_info(0)
        assert gi["lanes_per_row"] == 64 and gi["elems_per_lane"] == elems and gi["grid"] == 256, (rows, cols, gi)
        assert (f"CT = {tiles};" in p.group_source(0)), (rows, cols)
        p.destroy()


def test_which_tensors_are_accessed_non_temporally():
    # tensors of 32 MiB and more always; from 2 MiB on those no other kernel of the plan touches (a plan input one kernel
    # reads, a plan output nothing consumes); what several kernels read, and what is smaller, stays cacheable
    from workloads.patterns import batchnorm

    def flags(plan, k):
        src = plan.group_source(k)
        loads = re.findall(r"fs_load_row<\d+, V, NVL, L, NV, RAGGED, (true|false)>\(\w+, a\.p\[(\d+)\]", src)
        stores = re.findall(r"fs_store_row(?:_vec)?<\d+, V, NVL, L, NV, RAGGED, (true|false)>\(\w+, a\.p\[(\d+)\]", src)
        return [f for f, _ in loads], [f for f, _ in stores]

    p = fs.Plan(softmax_graph(4096, 1024))      # 16 MiB in, 16 MiB out, one kernel
    assert flags(p, 0) == (["true"], ["true"])
    p.destroy()
    p = fs.Plan(softmax_graph(256, 1024))       # 1 MiB: too small to matter
    assert flags(p, 0) == (["false"], ["false"])
    p.destroy()
    p = fs.Plan(batchnorm(4096, 1024))          # x (16 MiB) is read by all three kernels, y is written by the last
    assert p.stats()["num_launches"] == 3
    assert [flags(p, k) for k in range(3)] == [(["false"], []), (["false"], []), (["false"], ["true"])]
    p.destroy()
    p = fs.Plan(batchnorm(16384, 1024))         # 64 MiB: beyond the caches whoever reads it
    assert [flags(p, k)[0] for k in range(3)] == [["true"]] * 3
    p.destroy()


def test_recomputation_never_moves_more_bytes_than_the_same_groups_without_it():
    # random graphs, with and without views: the library's plan against the same grouping given back as the caller's
    # plan (which is taken as it is: every value on a kernel boundary is stored by its producer and read by its consumers)
    import sys
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from graphgen import random_graph
    fewer = 0
    for seed in range(3000, 3006):
        rows, cols = [(1000, 1000), (64, 16384), (4096, 260), (257, 1025)][seed % 4]
        g = random_graph(seed, rows, cols, 40, views=(seed % 2 == 0))
        p = fs.Plan(g)
        own = [max(k, 0) for k in p.node_groups()]
        q = fs.Plan(g, group_of_node=own)
        a, b = p.stats(), q.stats()
        assert a["num_launches"] == b["num_launches"] and a["launched_hbm_bytes"] <= b["launched_hbm_bytes"], (seed, a, b)
        assert p.workspace_bytes() <= q.workspace_bytes()
        fewer += a["launched_hbm_bytes"] < b["launched_hbm_bytes"]
        p.destroy()
        q.destroy()
    assert fewer >= 2


def test_survey_patterns_are_single_kernels():
    # every pattern of the shape survey (softmax variants, norms, optimizer update, column sums, transposes, backward passes)
    # from 64 to 131072 columns plans as ONE stitched kernel (the softmax over 8 rows of a million columns is the one
    # exception: cut into three kernels that each fill the device)
    # (and batch normalisation, whose column statistics cannot be broadcast back inside the kernel that folds them:
    # means, variances of the centred values, the normalised tensor -- x read three times and y written once)
    from workloads import patterns as survey
    for name, g, rows, cols in survey.cases() + survey.more_cases():
        p = fs.Plan(g)
        if rows <= 32 and cols >= (1 << 20) and "softmax" in name:
            assert p.stats()["num_launches"] == 3, (name, rows, cols)
        elif "batchnorm" in name:
            assert p.stats()["num_launches"] == 3, (name, rows, cols)
            assert p.stats()["launched_hbm_bytes"] == min_hbm_bytes(g) + 2 * rows * cols * 4 + 3 * cols * 4
        else:
            assert p.stats()["num_launches"] == 1, (name, rows, cols)
            assert p.stats()["launched_hbm_bytes"] == p.stats()["min_hbm_bytes"] == min_hbm_bytes(g)
        p.destroy()


# ------------------------------------------------------------------ boundary: statuses that need no GPU
def test_stats_report_the_unfused_traffic_of_the_same_dag():
    # fs_plan_stats' fourth figure is what one launch per compute node would move, whatever mode the plan was made in
    for g in (softmax_graph(256, 1024), layernorm_gelu_graph(512, 1024), multi_reduce_graph(4096, 512), random_dag_graph()):
        p, u = fs.Plan(g), fs.Plan(g, mode=fs.FS_MODE_UNFUSED)
        sp, su = p.stats(), u.stats()
        assert sp["unfused_hbm_bytes"] == su["unfused_hbm_bytes"] == su["launched_hbm_bytes"] > sp["launched_hbm_bytes"] >= sp["min_hbm_bytes"]
        p.destroy()
        u.destroy()
    # softmax by hand: max reads x, writes m; sub reads x, m, writes d; exp d -> e; sum e -> s; div e, s -> y
    R, C = 256, 1024
    full, vec = 4 * R * C, 4 * R
    p = fs.Plan(softmax_graph(R, C))
    assert p.stats()["unfused_hbm_bytes"] == (full + vec) + (full + vec + full) + 2 * full + (full + vec) + (full + vec + full)
    p.destroy()


def test_device_limits_without_a_device():
    import torch
    lim = fs.device_limits()
    if torch.cuda.is_available():
        assert lim["from_device"] and lim["compute_units"] > 0 and lim["lds_bytes_per_workgroup"] >= 65536
    else:   # the published MI355X figures stand in
        assert lim == {"compute_units": 256, "lds_bytes_per_workgroup": 163840, "resident_lanes": 524288, "l2_bytes": 4 << 20,
                       "from_device": False}
    # a budget above what one workgroup may use is refused, at the limit it is accepted
    assert _status(softmax_graph(64, 1024), lds_budget_bytes=lim["lds_bytes_per_workgroup"] + 1) == "FS_ERR_INVALID_ARG"
    assert _status(softmax_graph(64, 1024), lds_budget_bytes=lim["lds_bytes_per_workgroup"]) == "FS_OK"


def test_run_refuses_overlapping_buffers_before_touching_the_device():
    # Pointer checks come before any HIP call, so made-up addresses are enough.  Only calls that MUST be refused are
    # made (an accepted call would launch on those addresses), and only where no GPU is visible.
    import torch
    if torch.cuda.is_available():
        pytest.skip("host-only check: with a device present the accepted path would launch on made-up addresses")
    g = Graph()
    a, b = g.input(64, 256), g.input(64, 256)
    s = g.binary("add", a, b)
    t = g.transpose(g.binary("mul", s, a))       # two groups: the product crosses a group boundary through the workspace
    c = g.reduce_col("sum", s)
    g.set_outputs([s, t, c])
    p = fs.Plan(g)
    need = p.workspace_bytes()
    nb = 64 * 256 * 4
    base = 0x7000_0000_0000
    ins, outs, ws = [base, base + 2 * nb], [base + 4 * nb, base + 6 * nb, base + 8 * nb], base + 16 * nb

    def status(i, o, w=ws, wb=max(need, 256)):
        try:
            p.run(i, o, w, wb)
        except fs.FsError as e:
            return e.status_name, str(e)
        return "FS_OK", ""

    assert status([outs[0], ins[1]], outs)[0] == "FS_ERR_INVALID_ARG"                      # output 0 IS input 0
    assert "outputs[0] overlaps inputs[0]" in status([outs[0] - nb + 16, ins[1]], outs)[1]  # partial overlap from below
    assert "outputs[1] overlaps inputs[1]" in status([ins[0], outs[1] + nb - 16], outs)[1]  # partial overlap from above
    assert "outputs[1] overlaps outputs[0]" in status(ins, [outs[0], outs[0] + 16, outs[2]])[1]
    assert "outputs[2] overlaps outputs[1]" in status(ins, [outs[0], outs[1], outs[1] + nb - 16])[1]
    if need:
        assert "outputs[0] overlaps the workspace" in status(ins, [ws + 256, outs[1], outs[2]])[1]
        assert "inputs[1] overlaps the workspace" in status([ins[0], ws + need - 16], outs)[1]
        assert status(ins, outs, ws, need - 1)[0] == "FS_ERR_WORKSPACE"
        assert status(ins, outs, ws + 64)[0] == "FS_ERR_WORKSPACE"
    assert status([ins[0] + 4, ins[1]], outs)[0] == "FS_ERR_INVALID_ARG"                    # misaligned
    assert status([0, ins[1]], outs)[0] == "FS_ERR_INVALID_ARG"                             # NULL
    # inputs may alias each other (only read): not refused for that reason -> the call reaches the device query and fails THERE
    assert status([ins[0], ins[0]], outs)[0] == "FS_ERR_HIP"
    # loading needs a device
    with pytest.raises(fs.FsError) as e:
        p.load()
    assert e.value.status_name == "FS_ERR_HIP"
    p.destroy()


# ------------------------------------------------------------------ reshape / bitcast / concat
def _attention_scores_graph(b=2, h=3, s=64, d=32):
    """Per-head softmax of an N-D tensor [b, s, h*s] -> view [b*s*h, s], then back, with a concat on the way in."""
    g = Graph()
    x = g.input(b * s, h * s)                       # [b, s, h, s] stored row-major, seen as [b*s, h*s]
    bias = g.input(1, s)
    v = g.view_nd(x, (b, s, h, s), 3)               # [b*s*h, s]: one softmax row per (batch, position, head)
    z = g.binary("add", v, g.bcast_rowvec(bias, b * s * h))
    m = g.reduce_row("max", z)
    e = g.unary("exp", g.binary("sub", z, g.bcast_colvec(m, s)))
    y = g.binary("div", e, g.bcast_colvec(g.reduce_row("sum", e), s))
    out = g.reshape(y, b * s, h * s, op="bitcast")  # back to the caller's 2-D shape: a view, no copy
    g.set_outputs([out])
    return g


def test_views_cost_no_launch_and_no_copy():
    g = _attention_scores_graph()
    p = fs.Plan(g)
    st = p.stats()
    assert st["num_launches"] == 1 and st["launched_hbm_bytes"] == st["min_hbm_bytes"] == min_hbm_bytes(g)
    gi = p.group_info(0)
    assert (gi["dom_rows"], gi["dom_cols"]) == (2 * 64 * 3, 64) and p.workspace_bytes() == 0   # the view's shape is the work space
    groups = p.node_groups()
    assert all(groups[i] == -1 for i, n in enumerate(g.nodes) if n.op in ("reshape", "bitcast"))
    p.destroy()
    u = fs.Plan(g, mode=fs.FS_MODE_UNFUSED)
    assert u.stats()["num_launches"] == len(g.compute_ids()) == 6     # the two views are not launches
    u.destroy()
    # a reshape between two computations that both have a row structure separates them (the consumer's rows are not the
    # producer's) without a copy: the producer writes once, the consumer reads the same bytes under the other shape
    g2 = Graph()
    x = g2.input(128, 256)
    a = g2.binary("sub", x, g2.bcast_colvec(g2.reduce_row("max", x), 256))
    r = g2.reshape(a, 512, 64)
    s = g2.reduce_row("sum", r)
    g2.set_outputs([g2.binary("sub", r, g2.bcast_colvec(s, 64))])
    p = fs.Plan(g2)
    assert p.stats()["num_launches"] == 2 and p.workspace_bytes() >= 128 * 256 * 4
    assert p.stats()["launched_hbm_bytes"] == 4 * 128 * 256 * 4
    p.destroy()


def test_a_reshape_next_to_an_elementwise_region_is_fused_through():
    # Table 1: a Row schedule passes through a Reshape.  Dense row-major tensors make an elementwise region - no broadcast, no
    # reduction - the same computation under either shape, so it takes the shape of the other side of the view and shares its kernel.
    # up: an activation, a reshape, then a reduction over the NEW rows: one kernel in the new shape, the input read as it lies
    g = Graph()
    x, y = g.input(128, 256), g.input(128, 256)
    a = g.binary("mul", g.unary("tanh", x), y)
    r = g.reshape(a, 512, 64)
    s = g.reduce_row("sum", r)
    g.set_outputs([g.binary("sub", r, g.bcast_colvec(s, 64))])
    p = fs.Plan(g)
    gi = p.group_info(0)
    assert p.stats()["num_launches"] == 1 and p.workspace_bytes() == 0 and (gi["dom_rows"], gi["dom_cols"]) == (512, 64)
    assert p.stats()["launched_hbm_bytes"] == p.stats()["min_hbm_bytes"] == 3 * 128 * 256 * 4
    p.destroy()
    # down: a softmax over the old rows, a bitcast, then a residual add and an activation in the new shape: one kernel in the OLD shape
    g = Graph()
    x, res = g.input(96, 200), g.input(300, 64)
    e = g.unary("exp", g.binary("sub", x, g.bcast_colvec(g.reduce_row("max", x), 200)))
    sm = g.binary("div", e, g.bcast_colvec(g.reduce_row("sum", e), 200))
    v = g.reshape(sm, 300, 64, op="bitcast")
    g.set_outputs([g.unary("gelu_tanh", g.binary("add", v, res))])
    p = fs.Plan(g)
    gi = p.group_info(0)
    assert p.stats()["num_launches"] == 1 and p.workspace_bytes() == 0 and (gi["dom_rows"], gi["dom_cols"]) == (96, 200)
    p.destroy()
    # the unfused executor runs every op on its own either way
    u = fs.Plan(g, mode=fs.FS_MODE_UNFUSED)
    assert u.stats()["num_launches"] == len(g.compute_ids())
    u.destroy()
    # not through: the value is also needed under its old shape by something with a row structure, or a broadcast sits in the region
    g = Graph()
    x, w = g.input(128, 256), g.input(1, 256)
    a = g.binary("mul", g.unary("tanh", x), g.bcast_rowvec(w, 128))     # a per-column operand: tied to the old columns
    r = g.reshape(a, 512, 64)
    g.set_outputs([g.binary("sub", r, g.bcast_colvec(g.reduce_row("sum", r), 64))])
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 2
    p.destroy()
    # a region that ends in a plan output and a view of something else: both views absorbed, still one kernel
    g = Graph()
    x, y = g.input(64, 96), g.input(48, 128)
    a = g.unary("sigmoid", x)
    b = g.binary("add", g.reshape(a, 48, 128), y)
    g.set_outputs([g.reshape(g.unary("neg", b), 64, 96)])
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 1 and p.workspace_bytes() == 0
    p.destroy()


def test_view_and_concat_validation():
    g = Graph()
    x = g.input(4, 6)
    r = g.reshape(x, 3, 8)
    g.set_outputs([r])
    assert _status(g) == "FS_ERR_BAD_GRAPH"             # a view of a plan input computes nothing
    g = Graph()
    x = g.input(4, 6)
    y = g.unary("neg", x)
    g.set_outputs([y, g.reshape(y, 3, 8)])
    assert _status(g) == "FS_ERR_BAD_GRAPH"             # two views of one value as outputs: one buffer cannot be both
    g = Graph()
    x = g.input(4, 6)
    r = g.reshape(g.unary("neg", x), 3, 8)
    g.nodes[r].cols = 7
    g.set_outputs([r])
    assert _status(g) == "FS_ERR_SHAPE"
    g = Graph()
    x = g.input(4, 6)
    r = g.reshape(g.unary("neg", x), 3, 8)
    g.nodes[r].dtype = "bf16"
    g.set_outputs([r])
    assert _status(g) == "FS_ERR_DTYPE"
    g = Graph()
    v = g.input(1, 6)
    r = g.reshape(g.bcast_rowvec(v, 4), 3, 8)
    g.set_outputs([g.unary("neg", r)])
    assert _status(g) == "FS_ERR_BAD_GRAPH"             # a view of a broadcast, which is never materialised
    g = Graph()
    a, b = g.input(4, 6), g.input(4, 2)
    c = g.concat(a, b)
    g.nodes[c].cols = 9
    g.set_outputs([c])
    assert _status(g) == "FS_ERR_SHAPE"
    g = Graph()
    a, b = g.input(4, 6), g.input(4, 2, "bf16")
    c = g._add(type(g.nodes[0])("concat", "f32", 4, 8, (a, b), attr="cols"))
    g.set_outputs([c])
    assert _status(g) == "FS_ERR_DTYPE"


def test_concat_is_read_as_one_row_by_its_consumers():
    # two tensors from memory joined along columns and normalised: one kernel, nothing copied
    g = Graph()
    a, b = g.input(512, 96), g.input(512, 160)
    c = g.concat(a, b)
    m = g.reduce_row("mean", c)
    g.set_outputs([g.binary("sub", c, g.bcast_colvec(m, 256))])
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 1 and p.stats()["launched_hbm_bytes"] == min_hbm_bytes(g)
    assert "fs_load_row_concat" in p.group_source(0)
    gi = p.group_info(0)
    assert 96 % gi["vec_elems"] == 0
    p.destroy()
    # a seam at an odd column forces narrower accesses, not a wrong one
    g = Graph()
    a, b = g.input(64, 30), g.input(64, 34)
    g.set_outputs([g.unary("neg", g.concat(a, b))])
    p = fs.Plan(g)
    assert p.group_info(0)["vec_elems"] == 2
    p.destroy()
    # an operand computed by the graph is materialised first: producer | concat consumer
    g = Graph()
    a, b = g.input(64, 32), g.input(64, 32)
    c = g.concat(g.unary("tanh", a), b)
    g.set_outputs([g.reduce_row("sum", c)])
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 2
    p.destroy()
    # along rows
    g = Graph()
    a, b = g.input(100, 64), g.input(28, 64)
    g.set_outputs([g.reduce_row("max", g.unary("abs", g.concat(a, b, "rows")))])
    p = fs.Plan(g)
    assert p.stats()["num_launches"] == 1 and p.group_info(0)["dom_rows"] == 128
    p.destroy()
