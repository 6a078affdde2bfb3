"""The five synthetic workloads (DAG + seeded inputs).

They stand in for the patterns the paper optimises: the softmax pattern of its
motivating example (Section 2.1 / Section 5.1.3: Reduce.1 -> Exponential.1 ->
Reduce.2 -> Divide.1), normalisation chains, large elementwise layers (Section 3.2),
multi-root reductions (Section 4.3) and the reduce / transpose / elementwise
interplay it reports for its Speech workload (Section 6.3).

No arithmetic of the method lives here: builders only describe DAGs, and input
generators only draw seeded random numbers.  Both the CPU oracle and the GPU
library consume exactly these objects.
"""
from __future__ import annotations

import hashlib
from typing import Dict, List, Tuple

import numpy as np

from .graph import Graph

BASE_SEED = 181105213


def _seed(cfg: int, tensor_index: int) -> int:
    return BASE_SEED + 1000 * cfg + tensor_index


def _draw(rng: np.random.Generator, kind: str, rows: int, cols: int, a: float, b: float) -> np.ndarray:
    """fp64 draws -> affine -> fp32, generated in row chunks (same stream as one big draw)."""
    out = np.empty((rows, cols), dtype=np.float32)
    step = max(1, (1 << 22) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        if kind == "normal":      # mean a, std b
            blk = rng.standard_normal((r1 - r0, cols)) * b + a
        elif kind == "uniform":   # U(a, b)
            blk = rng.uniform(a, b, (r1 - r0, cols))
        else:
            raise ValueError(kind)
        out[r0:r1] = blk.astype(np.float32)
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as raw uint16 bits (inputs contain no NaN)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ---------------------------------------------------------------------------------------------
# cfg 1: softmax, 5 ops
# ---------------------------------------------------------------------------------------------
def softmax_graph(rows: int = 256, cols: int = 1024) -> Graph:
    g = Graph()
    x = g.input(rows, cols, "f32", "x")
    m = g.reduce_row("max", x, name="m")
    d = g.binary("sub", x, g.bcast_colvec(m, cols), name="d")
    e = g.unary("exp", d, name="e")
    s = g.reduce_row("sum", e, name="s")
    y = g.binary("div", e, g.bcast_colvec(s, cols), name="y")
    g.set_outputs([y])
    return g


def softmax_inputs(rows: int = 256, cols: int = 1024) -> List[np.ndarray]:
    return [_draw(np.random.default_rng(_seed(1, 0)), "normal", rows, cols, 0.0, 1.0)]


# ---------------------------------------------------------------------------------------------
# cfg 2: LayerNorm + bias + tanh-GeLU, bf16 in/out, fp32 arithmetic
# ---------------------------------------------------------------------------------------------
def layernorm_gelu_graph(rows: int = 16384, cols: int = 1024, eps: float = 1e-5, decomposed_gelu: bool = False) -> Graph:
    g = Graph()
    x = g.input(rows, cols, "bf16", "x")
    gamma = g.input(1, cols, "f32", "gamma")
    beta = g.input(1, cols, "f32", "beta")
    bias = g.input(1, cols, "f32", "bias")
    xf = g.unary("convert", x, "f32", name="xf")
    mu = g.reduce_row("mean", xf, name="mu")
    xc = g.binary("sub", xf, g.bcast_colvec(mu, cols), name="xc")
    sq = g.binary("mul", xc, xc, name="sq")
    var = g.reduce_row("mean", sq, name="var")
    ve = g.binary("add", var, g.const(eps, rows, 1), name="var_eps")
    rstd = g.unary("rsqrt", ve, name="rstd")
    xn = g.binary("mul", xc, g.bcast_colvec(rstd, cols), name="xn")
    xg = g.binary("mul", xn, g.bcast_rowvec(gamma, rows), name="xg")
    xb = g.binary("add", xg, g.bcast_rowvec(beta, rows), name="xb")
    z = g.binary("add", xb, g.bcast_rowvec(bias, rows), name="z")
    if not decomposed_gelu:
        act = g.unary("gelu_tanh", z, name="gelu")
    else:
        # 0.5 z (1 + tanh(k (z + c z^3))) spelled out in primitive ops
        z2 = g.binary("mul", z, z)
        z3 = g.binary("mul", z2, z)
        cz3 = g.binary("mul", z3, g.const(0.044715, rows, cols))
        inner = g.binary("add", z, cz3)
        kin = g.binary("mul", inner, g.const(0.7978845608028654, rows, cols))
        th = g.unary("tanh", kin)
        onep = g.binary("add", th, g.const(1.0, rows, cols))
        hz = g.binary("mul", z, g.const(0.5, rows, cols))
        act = g.binary("mul", hz, onep, name="gelu")
    out = g.unary("convert", act, "bf16", name="out")
    g.set_outputs([out])
    return g


def layernorm_gelu_inputs(rows: int = 16384, cols: int = 1024) -> List[np.ndarray]:
    x = _draw(np.random.default_rng(_seed(2, 0)), "normal", rows, cols, 0.0, 1.0)
    gamma = _draw(np.random.default_rng(_seed(2, 1)), "normal", 1, cols, 1.0, 0.1)
    beta = _draw(np.random.default_rng(_seed(2, 2)), "normal", 1, cols, 0.0, 0.1)
    bias = _draw(np.random.default_rng(_seed(2, 3)), "normal", 1, cols, 0.0, 0.02)
    return [f32_to_bf16_bits(x), gamma, beta, bias]


# ---------------------------------------------------------------------------------------------
# cfg 3: 20-op elementwise DAG, 4 inputs + 2 row vectors, 2 outputs
# ---------------------------------------------------------------------------------------------
def elementwise20_graph(rows: int = 65536, cols: int = 1024) -> Graph:
    g = Graph()
    a = g.input(rows, cols, "f32", "a")
    b = g.input(rows, cols, "f32", "b")
    c = g.input(rows, cols, "f32", "c")
    d = g.input(rows, cols, "f32", "d")
    u = g.input(1, cols, "f32", "u")
    v = g.input(1, cols, "f32", "v")
    U = g.bcast_rowvec(u, rows)
    V = g.bcast_rowvec(v, rows)
    n1 = g.binary("add", a, b, name="n1")
    n2 = g.binary("mul", c, U, name="n2")
    n3 = g.binary("sub", n1, n2, name="n3")
    n4 = g.unary("tanh", n3, name="n4")
    n5 = g.binary("mul", d, V, name="n5")
    n6 = g.unary("sigmoid", n5, name="n6")
    n7 = g.binary("mul", n4, n6, name="n7")
    n8 = g.binary("max", a, c, name="n8")
    n9 = g.binary("add", n7, n8, name="n9")
    n10 = g.binary("sub", b, d, name="n10")
    n11 = g.binary("mul", n10, n10, name="n11")
    n12 = g.unary("tanh", n11, name="n12")
    n13 = g.cmp("gt", n1, n2, name="n13")
    n14 = g.select(n13, n9, n12, name="n14")
    n15 = g.binary("add", n14, U, name="n15")
    n16 = g.unary("sigmoid", n15, name="n16")
    n17 = g.binary("mul", n16, n3, name="n17")
    n18 = g.binary("max", n17, n10, name="n18")
    n19 = g.binary("sub", n9, n18, name="n19")
    n20 = g.binary("add", n19, n12, name="n20")
    g.set_outputs([n17, n20])
    return g


def elementwise20_inputs(rows: int = 65536, cols: int = 1024) -> List[np.ndarray]:
    ins = [_draw(np.random.default_rng(_seed(3, k)), "uniform", rows, cols, -2.0, 2.0) for k in range(4)]
    ins += [_draw(np.random.default_rng(_seed(3, 4 + k)), "uniform", 1, cols, -1.0, 1.0) for k in range(2)]
    return ins


# ---------------------------------------------------------------------------------------------
# cfg 4: multi-output reduction from one read of x
# ---------------------------------------------------------------------------------------------
def multi_reduce_graph(rows: int = 65536, cols: int = 512) -> Graph:
    g = Graph()
    x = g.input(rows, cols, "f32", "x")
    q = g.binary("mul", x, x, name="q")
    cs = g.reduce_col("sum", x, name="colsum")
    cq = g.reduce_col("sum", q, name="colsumsq")
    rs = g.reduce_row("sum", q, name="rowsumsq")
    rn = g.unary("sqrt", rs, name="rownorm")
    g.set_outputs([cs, cq, rn])
    return g


def multi_reduce_inputs(rows: int = 65536, cols: int = 512) -> List[np.ndarray]:
    return [_draw(np.random.default_rng(_seed(4, 0)), "normal", rows, cols, 0.5, 1.0)]


# ---------------------------------------------------------------------------------------------
# cfg 5: seeded random DAG, 200 compute nodes on [512,k] tensors
# ---------------------------------------------------------------------------------------------
def random_dag_graph(num_nodes: int = 200, rows: int = 512, ks: Tuple[int, ...] = (64, 128, 256),
                     seed: int = BASE_SEED + 5000, num_sources: int = 6) -> Graph:
    """Node mix: 60% elementwise, 20% row-broadcast binary, 15% row reduce, 5% transpose.

    Shape classes: S_k = [rows,k], T_k = [k,rows], Rv = [rows,1], Kv_k = [k,1], Cv_k = [1,k].
    Instead of evaluating values, the generator carries a conservative magnitude bound per
    node and redraws any node whose bound exceeds 1e6, so no value can overflow.
    """
    rng = np.random.default_rng(seed)
    g = Graph()
    bound: Dict[int, float] = {}
    pools: Dict[Tuple[str, int], List[int]] = {}

    def pool(kind: str, k: int = 0) -> List[int]:
        return pools.setdefault((kind, k), [])

    while True:
        src_k = [int(ks[int(rng.integers(len(ks)))]) for _ in range(num_sources)]
        if set(src_k) == set(ks) or num_sources < len(ks):
            break
    for k in src_k:
        i = g.input(rows, k, "f32")
        bound[i] = 6.0
        pool("S", k).append(i)
    for k in ks:
        i = g.input(1, k, "f32")
        bound[i] = 6.0
        pool("Cv", k).append(i)

    def pick(lst: List[int]) -> int:
        j = min(int(rng.geometric(0.3)) - 1, len(lst) - 1)
        return lst[len(lst) - 1 - j]

    def full_classes() -> List[Tuple[str, int]]:
        return [key for key in pools if key[0] in ("S", "T") and pools[key]]

    def vec_classes() -> List[Tuple[str, int]]:
        return [key for key in pools if key[0] in ("Rv", "Kv", "Cv") and pools[key]]

    LIMIT = 1e6
    made = 0
    while made < num_nodes:
        r = rng.random()
        if r < 0.60:                                        # elementwise
            cands = full_classes()
            if vec_classes() and rng.random() < 0.1:
                cands = vec_classes()
            key = cands[int(rng.integers(len(cands)))]
            lst = pools[key]
            if rng.random() < 0.4:
                op = ("tanh", "sigmoid", "neg", "abs")[int(rng.integers(4))]
                a = pick(lst)
                nb = 1.0 if op in ("tanh", "sigmoid") else bound[a]
                node = g.unary(op, a)
            else:
                op = ("add", "sub", "mul", "max", "min")[int(rng.integers(5))]
                a = pick(lst)
                colv = pools.get(("Rv", 0), []) if key[0] == "S" else pools.get(("Kv", key[1]), []) if key[0] == "T" else []
                if colv and rng.random() < 0.25:
                    bsrc = pick(colv)
                    nb_b = bound[bsrc]
                    ncols = g.nodes[a].cols
                    mark = len(g.nodes)
                    b = g.bcast_colvec(bsrc, ncols)
                else:
                    mark = len(g.nodes)
                    b = pick(lst)
                    nb_b = bound[b]
                nb = bound[a] * nb_b if op == "mul" else (bound[a] + nb_b if op in ("add", "sub") else max(bound[a], nb_b))
                if nb > LIMIT:
                    del g.nodes[mark:]
                    continue
                node = g.binary(op, a, b)
            bound[node] = nb
            pools[key].append(node)
        elif r < 0.80:                                      # row-broadcast binary
            cands = [key for key in pools if key[0] == "S" and pools[key] and pools.get(("Cv", key[1]))]
            if not cands:
                continue
            key = cands[int(rng.integers(len(cands)))]
            a = pick(pools[key])
            vsrc = pick(pools[("Cv", key[1])])
            op = ("add", "sub", "mul", "max", "min")[int(rng.integers(5))]
            nb = bound[a] * bound[vsrc] if op == "mul" else (bound[a] + bound[vsrc] if op in ("add", "sub") else max(bound[a], bound[vsrc]))
            if nb > LIMIT:
                continue
            b = g.bcast_rowvec(vsrc, rows)
            node = g.binary(op, a, b)
            bound[node] = nb
            pools[key].append(node)
        elif r < 0.95:                                      # row reduce
            cands = full_classes()
            key = cands[int(rng.integers(len(cands)))]
            a = pick(pools[key])
            kind = ("sum", "max", "mean")[int(rng.integers(3))]
            nb = bound[a] * g.nodes[a].cols if kind == "sum" else bound[a]
            if nb > LIMIT:
                continue
            node = g.reduce_row(kind, a)
            bound[node] = nb
            if key[0] == "S":
                pool("Rv", 0).append(node)
            else:
                pool("Kv", key[1]).append(node)
        else:                                               # transpose
            cands = full_classes()
            key = cands[int(rng.integers(len(cands)))]
            a = pick(pools[key])
            node = g.transpose(a)
            bound[node] = bound[a]
            pool("T" if key[0] == "S" else "S", key[1]).append(node)
        made += 1

    used = set()
    for n in g.nodes:
        used.update(n.ins)
    sinks = [i for i in g.compute_ids() if i not in used]
    g.set_outputs(sinks)
    return g


def random_dag_inputs(g: Graph, cfg: int = 5) -> List[np.ndarray]:
    outs = []
    for t, i in enumerate(g.input_ids()):
        n = g.nodes[i]
        outs.append(_draw(np.random.default_rng(_seed(cfg, t)), "normal", n.rows, n.cols, 0.0, 1.0))
    return outs


# ---------------------------------------------------------------------------------------------
# ---------------------------------------------------------------------------------------------
# Backward-pass patterns (row reductions and column reductions in one subgraph).  Not among the
# five configurations of the headline benchmark: a second family for the same stitcher.
# cfg 6: LayerNorm backward: dx, dgamma, dbeta from x, dy, gamma
# cfg 7: softmax backward: dx = y * (dy - rowsum(dy * y))
# ---------------------------------------------------------------------------------------------
def layernorm_grad_graph(rows: int = 16384, cols: int = 1024, eps: float = 1e-5) -> Graph:
    g = Graph()
    x = g.input(rows, cols, "f32", "x")
    dy = g.input(rows, cols, "f32", "dy")
    gamma = g.input(1, cols, "f32", "gamma")
    mu = g.reduce_row("mean", x, name="mu")
    xc = g.binary("sub", x, g.bcast_colvec(mu, cols), name="xc")
    var = g.reduce_row("mean", g.binary("mul", xc, xc), name="var")
    rstd = g.unary("rsqrt", g.binary("add", var, g.const(eps, rows, 1)), name="rstd")
    xhat = g.binary("mul", xc, g.bcast_colvec(rstd, cols), name="xhat")
    dbeta = g.reduce_col("sum", dy, name="dbeta")
    dgamma = g.reduce_col("sum", g.binary("mul", dy, xhat), name="dgamma")
    gy = g.binary("mul", dy, g.bcast_rowvec(gamma, rows), name="gy")
    m1 = g.reduce_row("mean", gy, name="m1")
    m2 = g.reduce_row("mean", g.binary("mul", gy, xhat), name="m2")
    t = g.binary("sub", gy, g.bcast_colvec(m1, cols))
    t = g.binary("sub", t, g.binary("mul", xhat, g.bcast_colvec(m2, cols)))
    dx = g.binary("mul", t, g.bcast_colvec(rstd, cols), name="dx")
    g.set_outputs([dx, dgamma, dbeta])
    return g


def layernorm_grad_inputs(rows: int = 16384, cols: int = 1024) -> List[np.ndarray]:
    return [_draw(np.random.default_rng(_seed(6, 0)), "normal", rows, cols, 0.0, 1.0),
            _draw(np.random.default_rng(_seed(6, 1)), "normal", rows, cols, 0.0, 1.0),
            _draw(np.random.default_rng(_seed(6, 2)), "normal", 1, cols, 1.0, 0.1)]


def softmax_grad_graph(rows: int = 16384, cols: int = 1024) -> Graph:
    g = Graph()
    y = g.input(rows, cols, "f32", "y")
    dy = g.input(rows, cols, "f32", "dy")
    s = g.reduce_row("sum", g.binary("mul", dy, y), name="s")
    dx = g.binary("mul", y, g.binary("sub", dy, g.bcast_colvec(s, cols)), name="dx")
    g.set_outputs([dx])
    return g


def softmax_grad_inputs(rows: int = 16384, cols: int = 1024) -> List[np.ndarray]:
    # y: positive rows of mean 1/cols (the scale of a softmax output; exact normalisation is not needed here)
    y = _draw(np.random.default_rng(_seed(7, 0)), "uniform", rows, cols, 0.0, 2.0 / cols)
    return [y, _draw(np.random.default_rng(_seed(7, 1)), "normal", rows, cols, 0.0, 1.0)]


def workload(cfg: int, rows: int | None = None) -> Tuple[Graph, List[np.ndarray], str]:
    """(graph, inputs, name) of workload cfg in 1..7 (1-5: the benchmark's; 6-7: backward patterns); `rows` resizes it."""
    if cfg == 1:
        r = rows or 256
        return softmax_graph(r, 1024), softmax_inputs(r, 1024), f"softmax_f32_{r}x1024"
    if cfg == 2:
        r = rows or 16384
        return layernorm_gelu_graph(r, 1024), layernorm_gelu_inputs(r, 1024), f"layernorm_bias_gelu_bf16_{r}x1024"
    if cfg == 3:
        r = rows or 65536
        return elementwise20_graph(r, 1024), elementwise20_inputs(r, 1024), f"elementwise20_f32_{r}x1024"
    if cfg == 4:
        r = rows or 65536
        return multi_reduce_graph(r, 512), multi_reduce_inputs(r, 512), f"multi_reduce_f32_{r}x512"
    if cfg == 5:
        g = random_dag_graph(rows=rows or 512)
        return g, random_dag_inputs(g), f"random_dag200_{rows or 512}xk"
    if cfg == 6:
        r = rows or 16384
        return layernorm_grad_graph(r, 1024), layernorm_grad_inputs(r, 1024), f"layernorm_grad_f32_{r}x1024"
    if cfg == 7:
        r = rows or 16384
        return softmax_grad_graph(r, 1024), softmax_grad_inputs(r, 1024), f"softmax_grad_f32_{r}x1024"
    raise ValueError(cfg)


def sha256_of(arrays: List[np.ndarray]) -> str:
    h = hashlib.sha256()
    for a in arrays:
        h.update(np.ascontiguousarray(a).tobytes())
    return h.hexdigest()
