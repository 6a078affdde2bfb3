"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU oracle and of the library's host side (plan
ingestion, grouping, schedule / LDS planning, code generation), run on the benchmark DAGs, random graphs and
plans with views and concats.  Host code only: device code never runs under a sanitizer here."""
import os
import shutil
import subprocess
import sys

import pytest

import oracle.binding as ob
from paper_1811_05213_amd import binding as fb
from workloads import (Graph, layernorm_gelu_graph, layernorm_grad_graph, multi_reduce_graph, random_dag_graph, softmax_graph,
                       elementwise20_graph)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "san")
FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", LD_PRELOAD="")


def _write_plan(graph, path, opc, dt, cmp_, red, axis):
    with open(path, "w") as f:
        f.write(f"{len(graph.nodes)} {len(graph.outputs)}\n")
        for n in graph.nodes:
            ins = list(n.ins) + [0] * (3 - len(n.ins))
            attr = cmp_[n.attr] if n.op == "cmp" else red[n.attr] if n.op.startswith("reduce") else axis[n.attr] if n.op == "concat" else 0
            f.write(f"{opc[n.op]} {dt[n.dtype]} {n.rows} {n.cols} {len(n.ins)} {ins[0]} {ins[1]} {ins[2]} {attr} {n.value!r}\n")
        f.write(" ".join(map(str, graph.outputs)) + "\n")


def _graphs():
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from graphgen import random_graph
    out = [("softmax", softmax_graph(40, 200)), ("layernorm", layernorm_gelu_graph(33, 520)), ("ew20", elementwise20_graph(20, 64)),
           ("multi", multi_reduce_graph(300, 36)), ("lngrad", layernorm_grad_graph(50, 130)), ("dag", random_dag_graph(rows=64, ks=(8, 24, 40)))]
    out += [(f"rand{seed}", random_graph(seed, r, c)) for seed, r, c in ((1, 37, 72), (6, 129, 34), (9, 65, 63))]
    # ... and with reshapes / bitcasts / concats, which the planner's view-absorbing pass rewrites
    out += [(f"randv{seed}", random_graph(seed, r, c, 35, views=True)) for seed, r, c in ((1000, 65, 63), (1004, 40, 200), (1017, 12, 330), (1076, 96, 26))]
    g = Graph()
    a, b, w = g.input(24, 20), g.input(24, 12), g.input(1, 96)
    c = g.concat(a, b)
    v = g.reshape(c, 8, 96)
    t = g.binary("mul", v, g.bcast_rowvec(w, 8))
    s = g.reduce_row("sum", t)
    g.set_outputs([g.reshape(g.binary("sub", t, g.bcast_colvec(s, 96)), 24, 32, op="bitcast"), g.concat(g.unary("neg", a), a, "rows")])
    out.append(("views", g))
    return out


@pytest.fixture(scope="module")
def workdir(tmp_path_factory):
    if not shutil.which("gcc") or not shutil.which("g++"):
        pytest.skip("no host compiler")
    d = tmp_path_factory.mktemp("san")
    return str(d)


def test_oracle_under_address_and_ub_sanitizers(workdir):
    exe = os.path.join(workdir, "oracle_san")
    subprocess.run(["gcc", "-std=c99", "-fopenmp", "-ffp-contract=off", "-Wall"] + FLAGS +
                   [os.path.join(ROOT, "oracle", "fso.c"), os.path.join(SAN, "oracle_san_main.c"), "-o", exe, "-lm"], check=True)
    files = []
    for name, g in _graphs():
        p = os.path.join(workdir, f"o_{name}.plan")
        _write_plan(g, p, ob._OPC, ob._DT, ob._CMP, ob._RED, ob._AXIS)
        files.append(p)
    r = subprocess.run([exe] + files, env=ENV, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "oracle ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])


def test_host_planner_under_address_and_ub_sanitizers(workdir):
    exe = os.path.join(workdir, "planner_san")
    csrc = os.path.join(ROOT, "paper_1811_05213_amd", "csrc")
    srcs = [os.path.join(csrc, f) for f in ("fs_graph.cpp", "fs_group.cpp", "fs_codegen.cpp", "fs_perflib.cpp")]
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wno-unused-function"] + FLAGS + ["-I" + os.path.join(ROOT, "include"), "-I" + csrc, "-I" + SAN] +
                   srcs + [os.path.join(SAN, "planner_san_main.cpp"), "-o", exe, "-ldl"], check=True)
    files = []
    for name, g in _graphs():
        p = os.path.join(workdir, f"p_{name}.plan")
        _write_plan(g, p, fb.OPCODE, fb.DTYPE, fb.CMP, fb.RED, fb.AXIS)
        files.append(p)
    r = subprocess.run([exe] + files, env=ENV, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-4000:])
    assert r.stdout.count("status 0") >= 3 * len(files), r.stdout   # every plan is planned in the three modes
