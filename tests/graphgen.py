"""Random fused-subgraph generator for parity sweeps: a richer op mix than the benchmark's DAG generator
(all unary ops, comparisons and selects, bf16 round trips, row and column reductions of every kind,
transposes, both kinds of broadcast).  Values stay tame by construction: unbounded ops are fed through
tanh / sigmoid / abs+const first, so no draw can overflow or leave an op's domain."""
from __future__ import annotations

import numpy as np

from workloads import Graph, f32_to_bf16_bits


def random_graph(seed: int, rows: int, cols: int, num_ops: int = 40):
    rng = np.random.default_rng(seed)
    g = Graph()
    # pools of f32 node ids by shape class
    full = [g.input(rows, cols), g.input(rows, cols, "bf16")]
    full[1] = g.unary("convert", full[1], "f32")
    flipped = [g.input(cols, rows)]
    colv = [g.input(rows, 1)]
    rowv = [g.input(1, cols)]
    preds = []
    # values whose bits are reproducible (inputs and correctly rounded ops of such values): only these feed comparisons,
    # because a predicate downstream of a 1-ulp transcendental may legitimately differ between two correct implementations
    exact = list(full)

    def bounded(x):  # |value| <= 1
        return g.unary("tanh" if rng.random() < 0.5 else "sigmoid", x)

    def positive(x, r, c):  # >= 0.5
        return g.binary("add", g.unary("abs", x), g.const(0.5, r, c))

    def pick(pool):
        return pool[int(rng.integers(len(pool)))]

    for _ in range(num_ops):
        kind = rng.choice(["unary", "binary", "bcast", "cmpsel", "bf16", "rrow", "rcol", "transpose", "vec"],
                          p=[0.22, 0.22, 0.14, 0.08, 0.06, 0.1, 0.06, 0.06, 0.06])
        if kind == "unary":
            x = pick(full)
            op = rng.choice(["neg", "abs", "exp", "log", "tanh", "sigmoid", "sqrt", "rsqrt", "rcp", "gelu_tanh"])
            if op == "exp":
                x = bounded(x)
            elif op in ("log", "sqrt", "rsqrt", "rcp"):
                x = positive(bounded(x), rows, cols)
            full.append(g.unary(op, x))
        elif kind == "binary":
            a, b = bounded(pick(full)), bounded(pick(full))
            op = rng.choice(["add", "sub", "mul", "div", "max", "min"])
            if op == "div":
                b = positive(b, rows, cols)
            full.append(g.binary(op, a, b))
        elif kind == "bcast":
            a = bounded(pick(full))
            if rng.random() < 0.5:
                full.append(g.binary(rng.choice(["add", "mul", "sub"]), a, g.bcast_rowvec(bounded(pick(rowv)), rows)))
            else:
                full.append(g.binary(rng.choice(["add", "mul", "sub"]), a, g.bcast_colvec(bounded(pick(colv)), cols)))
        elif kind == "cmpsel":
            a, b = pick(exact), pick(exact)
            if rng.random() < 0.5:
                exact.append(g.binary(rng.choice(["add", "sub", "mul", "max", "min"]), a, b))
                full.append(exact[-1])
                a = exact[-1]
            p = g.cmp(rng.choice(["gt", "ge", "lt", "le", "eq", "ne"]), a, b)
            preds.append(p)
            full.append(g.select(p, bounded(a), bounded(pick(full))))
        elif kind == "bf16":
            full.append(g.unary("convert", g.unary("convert", bounded(pick(full)), "bf16"), "f32"))
        elif kind == "rrow":
            colv.append(g.reduce_row(rng.choice(["sum", "max", "min", "mean"]), bounded(pick(full))))
        elif kind == "rcol":
            rowv.append(g.reduce_col(rng.choice(["sum", "max", "min", "mean"]), bounded(pick(full))))
        elif kind == "transpose":
            if rng.random() < 0.5:
                flipped.append(g.transpose(bounded(pick(full))))
            else:
                full.append(g.transpose(bounded(pick(flipped))))
        else:  # vector arithmetic
            if rng.random() < 0.5:
                colv.append(g.binary("add", bounded(pick(colv)), bounded(pick(colv))))
            else:
                rowv.append(g.binary("mul", bounded(pick(rowv)), bounded(pick(rowv))))
    used = set()
    for n in g.nodes:
        used.update(n.ins)
    free = ("input", "const", "bcast_rowvec", "bcast_colvec")
    sinks = [i for i, n in enumerate(g.nodes) if i not in used and n.op not in free]
    # a few interior values and a predicate leave as well; one output in bf16
    extra = [int(x) for x in rng.choice(full[2:] if len(full) > 2 else full, size=min(3, max(1, len(full) - 2)), replace=False)]
    outs = list(dict.fromkeys(sinks + extra + preds[:1]))
    outs = [o for o in outs if g.nodes[o].op not in free]
    g.set_outputs(outs)
    return g


def random_inputs(g: Graph, seed: int):
    rng = np.random.default_rng(seed + 77)
    out = []
    for i in g.input_ids():
        n = g.nodes[i]
        a = rng.standard_normal((n.rows, n.cols)).astype(np.float32)
        out.append(f32_to_bf16_bits(a) if n.dtype == "bf16" else a)
    return out
