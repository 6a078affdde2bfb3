"""Random fused-subgraph generator for parity sweeps: a richer op mix than the benchmark's DAG generator
(all unary ops, comparisons and selects, bf16 round trips, row and column reductions of every kind,
transposes, both kinds of broadcast).  Values stay tame by construction: unbounded ops are fed through
tanh / sigmoid / abs+const first, so no draw can overflow or leave an op's domain."""
from __future__ import annotations

import numpy as np

from workloads import Graph, f32_to_bf16_bits


def random_graph(seed: int, rows: int, cols: int, num_ops: int = 40, views: bool = False):
    """views=True adds the shape-modulation ops: reshapes / bitcasts to another factorisation of the same elements (with
    elementwise work and row reductions in that other shape, and the way back), and concats along columns and rows.
    (A switch, not a change of the op mix: graphs of seeds generated without it stay what they were.)"""
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

    # the other factorisation of rows*cols elements that views lead to, and the halves that concats join
    if cols % 2 == 0 and cols >= 2:
        alt_shape = (rows * 2, cols // 2)
    elif rows % 2 == 0:
        alt_shape = (rows // 2, cols * 2)
    else:
        alt_shape = (1, rows * cols)
    alt = []     # values of shape alt_shape
    outs_extra = []
    for _ in range(num_ops):
        if views and rng.random() < 0.18:
            which = rng.choice(["there", "work", "back", "ccols", "crows"])
            name = "bitcast" if rng.random() < 0.3 else "reshape"
            if which == "there" or (which in ("work", "back") and not alt):
                alt.append(g.reshape(bounded(pick(full)), alt_shape[0], alt_shape[1], op=name))
            elif which == "work":  # arithmetic and a row reduction in the other shape
                a = bounded(pick(alt))
                b = g.input(alt_shape[0], alt_shape[1]) if rng.random() < 0.5 else pick(alt)
                t = g.binary(rng.choice(["add", "mul", "sub"]), a, bounded(b))
                if rng.random() < 0.5:
                    r = g.reduce_row(rng.choice(["sum", "max", "mean"]), t)
                    outs_extra.append(r)
                    t = g.binary("sub", t, g.bcast_colvec(bounded(r), alt_shape[1]))
                alt.append(t)
            elif which == "back":
                full.append(g.reshape(pick(alt), rows, cols, op=name))
            elif which == "ccols" and cols >= 2:
                c0 = int(rng.integers(1, cols))
                if rng.random() < 0.5 and cols >= 8:
                    c0 = max(4, (c0 // 4) * 4) if c0 >= 4 else 4  # a seam that vector accesses can respect
                    c0 = min(c0, cols - 1)
                left = bounded(g.input(rows, c0)) if rng.random() < 0.5 else g.input(rows, c0)
                right = g.input(rows, cols - c0)
                full.append(g.concat(left, right, "cols"))
            elif which == "crows" and rows >= 2:
                r0 = int(rng.integers(1, rows))
                top = g.input(r0, cols)
                bottom = g.unary("tanh", g.input(rows - r0, cols)) if rng.random() < 0.5 else g.input(rows - r0, cols)
                full.append(g.concat(top, bottom, "rows"))
            else:
                full.append(g.unary("neg", bounded(pick(full))))
            continue
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
    sinks += [o for o in outs_extra if o not in sinks]
    # a few interior values and a predicate leave as well; one output in bf16
    extra = [int(x) for x in rng.choice(full[2:] if len(full) > 2 else full, size=min(3, max(1, len(full) - 2)), replace=False)]
    outs = list(dict.fromkeys(sinks + extra + preds[:1]))
    outs = [o for o in outs if g.nodes[o].op not in free]
    # (a value and a view of it, or two views of one value, cannot both be plan outputs: they would be one buffer)
    def root(o):
        while g.nodes[o].op in ("reshape", "bitcast"):
            o = g.nodes[o].ins[0]
        return o
    seen, kept = set(), []
    for o in outs:
        if root(o) in seen or g.nodes[root(o)].op in free:
            continue
        seen.add(root(o))
        kept.append(o)
    g.set_outputs(kept)
    return g


def random_inputs(g: Graph, seed: int):
    rng = np.random.default_rng(seed + 77)
    out = []
    for i in g.input_ids():
        n = g.nodes[i]
        a = rng.standard_normal((n.rows, n.cols)).astype(np.float32)
        out.append(f32_to_bf16_bits(a) if n.dtype == "bf16" else a)
    return out
