"""The allocation-free entry point (fs_plan_run_static) against fs_plan_run, through the C ABI.

Collected last on purpose: a failure here must not hide any other GPU test from `pytest -x`.
"""
import numpy as np
import pytest

import paper_1811_05213_amd as fs
from paper_1811_05213_amd.binding import FS_STATIC_SCRATCH_BYTES
from paper_1811_05213_amd.runner import DeviceRun
from workloads import Graph, layernorm_grad_graph, layernorm_grad_inputs, multi_reduce_graph, multi_reduce_inputs, random_dag_graph, random_dag_inputs

pytestmark = pytest.mark.gpu


def _both(graph, ins):
    """Outputs of fs_plan_run (caller's workspace) and of fs_plan_run_static (the library's static scratch), same plan."""
    import torch
    plan = fs.Plan(graph)
    assert 0 < plan.workspace_bytes() <= FS_STATIC_SCRATCH_BYTES
    r = DeviceRun(plan)
    r.set_inputs(ins)
    r.launch()
    want = r.results()
    for t in r.outputs:
        t.zero_()
    plan.load()
    stream = torch.cuda.current_stream().cuda_stream
    plan.run_static([t.data_ptr() for t in r.inputs], [t.data_ptr() for t in r.outputs], stream)
    got = r.results()
    plan.destroy()
    return want, got


def _same(want, got, what):
    # the kernels, their launch shapes and their fold orders are the same: the results are bit-identical
    for k, (w, g) in enumerate(zip(want, got)):
        np.testing.assert_array_equal(g.view(np.uint8), w.view(np.uint8), err_msg=f"{what}: output {k}")


def test_static_scratch_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    # column partials + tickets in the scratch; the second call is a smaller plan (other offsets inside the same array),
    # the third a multi-kernel plan whose boundary tensors live there too, the fourth the first one again
    cases = [("multi reduce 3000x512", multi_reduce_graph(3000, 512), multi_reduce_inputs(3000, 512)),
             ("multi reduce 700x512", multi_reduce_graph(700, 512), multi_reduce_inputs(700, 512)),
             ("random dag", None, None),
             ("layernorm backward 1000x1024", layernorm_grad_graph(1000, 1024), layernorm_grad_inputs(1000, 1024)),
             ("multi reduce 3000x512 again", multi_reduce_graph(3000, 512), multi_reduce_inputs(3000, 512))]
    for what, g, ins in cases:
        if g is None:
            g = random_dag_graph(num_nodes=120, rows=512, ks=(64, 128, 256), seed=13)
            ins = random_dag_inputs(g)
        want, got = _both(g, ins)
        _same(want, got, what)


def test_static_scratch_refuses_what_it_cannot_hold_and_plans_that_are_not_loaded():
    import torch
    # a plan that is not loaded: the entry point must not load (allocate) by itself
    g = multi_reduce_graph(900, 512)
    plan = fs.Plan(g)
    r = DeviceRun(plan)
    r.set_inputs(multi_reduce_inputs(900, 512))
    with pytest.raises(fs.FsError) as e:
        plan.run_static([t.data_ptr() for t in r.inputs], [t.data_ptr() for t in r.outputs])
    assert e.value.status_name == "FS_ERR_INVALID_ARG" and "fs_plan_load" in str(e.value)
    plan.destroy()
    # a workspace beyond the static array's size
    # (one kernel per op: the 16 MiB intermediate crosses a kernel boundary and lives in the workspace)
    big = Graph()
    x = big.input(4096, 1024)
    big.set_outputs([big.unary("neg", big.unary("exp", x))])
    plan = fs.Plan(big, mode=fs.FS_MODE_UNFUSED)
    assert plan.workspace_bytes() > FS_STATIC_SCRATCH_BYTES
    plan.load()
    xs = torch.zeros((4096, 1024), dtype=torch.float32, device="cuda:0")
    outs = [torch.empty((4096, 1024), dtype=torch.float32, device="cuda:0")]
    with pytest.raises(fs.FsError) as e:
        plan.run_static([xs.data_ptr()], [o.data_ptr() for o in outs])
    assert e.value.status_name == "FS_ERR_WORKSPACE" and "static scratch" in str(e.value)
    plan.destroy()
