"""Common fused patterns beyond the five benchmark workloads, as DAG builders (no arithmetic here: op names and shapes).

softmax variants, normalisations, an optimizer update, column sums, a bias gradient, transposes and backward passes:
the shapes `bench.py --survey` times and the planner tests walk through.  `cases()` lists (name, graph, rows, cols).
"""
from __future__ import annotations

from .configs import layernorm_gelu_graph, layernorm_grad_graph, softmax_graph, softmax_grad_graph
from .graph import Graph


def _f32(g, x, dt):
    return g.unary("convert", x, "f32") if dt != "f32" else x


def _out(g, y, dt):
    return g.unary("convert", y, dt) if dt != "f32" else y


def rmsnorm(r, c, dt="bf16"):
    g = Graph()
    x, w = g.input(r, c, dt), g.input(1, c)
    xf = _f32(g, x, dt)
    rs = g.unary("rsqrt", g.binary("add", g.reduce_row("mean", g.binary("mul", xf, xf)), g.const(1e-6, r, 1)))
    g.set_outputs([_out(g, g.binary("mul", g.binary("mul", xf, g.bcast_colvec(rs, c)), g.bcast_rowvec(w, r)), dt)])
    return g


def bias_gelu(r, c, dt="bf16"):
    g = Graph()
    x, b = g.input(r, c, dt), g.input(1, c)
    g.set_outputs([_out(g, g.unary("gelu_tanh", g.binary("add", _f32(g, x, dt), g.bcast_rowvec(b, r))), dt)])
    return g


def add_layernorm(r, c, dt="bf16"):
    g = Graph()
    x, res, gam, bet = g.input(r, c, dt), g.input(r, c, dt), g.input(1, c), g.input(1, c)
    h = g.binary("add", _f32(g, x, dt), _f32(g, res, dt))
    hc = g.binary("sub", h, g.bcast_colvec(g.reduce_row("mean", h), c))
    rstd = g.unary("rsqrt", g.binary("add", g.reduce_row("mean", g.binary("mul", hc, hc)), g.const(1e-5, r, 1)))
    y = g.binary("add", g.binary("mul", g.binary("mul", hc, g.bcast_colvec(rstd, c)), g.bcast_rowvec(gam, r)), g.bcast_rowvec(bet, r))
    g.set_outputs([_out(g, h, dt), _out(g, y, dt)])
    return g


def masked_softmax(r, c, dt="bf16"):
    g = Graph()
    x, m = g.input(r, c, dt), g.input(r, c, dt)
    z = g.binary("add", g.binary("mul", _f32(g, x, dt), g.const(0.125, r, c)), _f32(g, m, dt))
    e = g.unary("exp", g.binary("sub", z, g.bcast_colvec(g.reduce_row("max", z), c)))
    g.set_outputs([_out(g, g.binary("div", e, g.bcast_colvec(g.reduce_row("sum", e), c)), dt)])
    return g


def adam(r, c):
    g = Graph()
    p, gr, m, v = (g.input(r, c) for _ in range(4))
    k = lambda val: g.const(val, r, c)
    m2 = g.binary("add", g.binary("mul", m, k(0.9)), g.binary("mul", gr, k(0.1)))
    v2 = g.binary("add", g.binary("mul", v, k(0.999)), g.binary("mul", g.binary("mul", gr, gr), k(0.001)))
    upd = g.binary("div", m2, g.binary("add", g.unary("sqrt", v2), k(1e-8)))
    g.set_outputs([g.binary("sub", p, g.binary("mul", upd, k(1e-3))), m2, v2])
    return g


def colsum(r, c, dt="f32"):
    g = Graph()
    g.set_outputs([g.reduce_col("sum", _f32(g, g.input(r, c, dt), dt))])
    return g


def bias_grad(r, c):
    g = Graph()
    x, dy = g.input(r, c), g.input(r, c)
    t = g.binary("mul", dy, g.unary("tanh", x))
    g.set_outputs([t, g.reduce_col("sum", t)])
    return g


def transpose(r, c, dt="f32"):
    g = Graph()
    g.set_outputs([g.transpose(g.input(r, c, dt))])
    return g


def row_norms(r, c):
    g = Graph()
    x = g.input(r, c)
    g.set_outputs([g.unary("sqrt", g.reduce_row("sum", g.binary("mul", x, x))), g.reduce_row("max", x)])
    return g


def dropout_residual(r, c, dt="bf16"):
    g = Graph()
    x, res, m = g.input(r, c, dt), g.input(r, c, dt), g.input(r, c, "u8")
    kept = g.select(m, g.binary("mul", _f32(g, x, dt), g.const(1.0 / 0.9, r, c)), g.const(0.0, r, c))
    g.set_outputs([_out(g, g.binary("add", kept, _f32(g, res, dt)), dt)])
    return g


def batchnorm(r, c):
    """Training-mode batch normalisation over the rows of [r, c]: column statistics, then the normalised tensor."""
    g = Graph()
    x, gam, bet = g.input(r, c), g.input(1, c), g.input(1, c)
    mean = g.reduce_col("mean", x)
    xc = g.binary("sub", x, g.bcast_rowvec(mean, r))
    var = g.reduce_col("mean", g.binary("mul", xc, xc))
    rstd = g.unary("rsqrt", g.binary("add", var, g.const(1e-5, 1, c)))
    y = g.binary("add", g.binary("mul", g.binary("mul", xc, g.bcast_rowvec(rstd, r)), g.bcast_rowvec(gam, r)), g.bcast_rowvec(bet, r))
    g.set_outputs([y, mean, var])
    return g


def heads_softmax(r, c, head, dt="bf16"):
    """Softmax over `head` consecutive columns at a time: [r, c] viewed as [r*c/head, head] and back."""
    g = Graph()
    x = g.input(r, c, dt)
    v = g.reshape(x, r * c // head, head)
    z = _f32(g, v, dt)
    e = g.unary("exp", g.binary("sub", z, g.bcast_colvec(g.reduce_row("max", z), head)))
    y = _out(g, g.binary("div", e, g.bcast_colvec(g.reduce_row("sum", e), head)), dt)
    g.set_outputs([g.reshape(y, r, c)])
    return g


def concat_layernorm(r, c, dt="bf16"):
    g = Graph()
    a, b, gam, bet = g.input(r, c // 2, dt), g.input(r, c // 2, dt), g.input(1, c), g.input(1, c)
    h = _f32(g, g.concat(a, b, "cols"), dt)
    hc = g.binary("sub", h, g.bcast_colvec(g.reduce_row("mean", h), c))
    rstd = g.unary("rsqrt", g.binary("add", g.reduce_row("mean", g.binary("mul", hc, hc)), g.const(1e-5, r, 1)))
    y = g.binary("add", g.binary("mul", g.binary("mul", hc, g.bcast_colvec(rstd, c)), g.bcast_rowvec(gam, r)), g.bcast_rowvec(bet, r))
    g.set_outputs([_out(g, y, dt)])
    return g


def l2_normalise(r, c):
    g = Graph()
    x = g.input(r, c)
    inv = g.unary("rsqrt", g.binary("add", g.reduce_row("sum", g.binary("mul", x, x)), g.const(1e-12, r, 1)))
    g.set_outputs([g.binary("mul", x, g.bcast_colvec(inv, c))])
    return g


def bias_transpose(r, c, dt="bf16"):
    g = Graph()
    x, b = g.input(r, c, dt), g.input(1, c)
    g.set_outputs([g.transpose(_out(g, g.binary("add", _f32(g, x, dt), g.bcast_rowvec(b, r)), dt))])
    return g


def gelu_grad(r, c, dt="bf16"):
    """dy * d/dx gelu_tanh(x), written out in elementwise ops."""
    g = Graph()
    x, dy = g.input(r, c, dt), g.input(r, c, dt)
    xf, k = _f32(g, x, dt), (lambda val: g.const(val, r, c))
    x2 = g.binary("mul", xf, xf)
    t = g.unary("tanh", g.binary("mul", g.binary("mul", xf, k(0.7978845608)), g.binary("add", k(1.0), g.binary("mul", x2, k(0.044715)))))
    dt_dx = g.binary("mul", g.binary("mul", g.binary("sub", k(1.0), g.binary("mul", t, t)), k(0.7978845608)),
                     g.binary("add", k(1.0), g.binary("mul", x2, k(3 * 0.044715))))
    d = g.binary("add", g.binary("mul", k(0.5), g.binary("add", k(1.0), t)), g.binary("mul", g.binary("mul", k(0.5), xf), dt_dx))
    g.set_outputs([_out(g, g.binary("mul", _f32(g, dy, dt), d), dt)])
    return g


def logsumexp(r, c):
    g = Graph()
    x = g.input(r, c)
    m = g.reduce_row("max", x)
    s = g.reduce_row("sum", g.unary("exp", g.binary("sub", x, g.bcast_colvec(m, c))))
    g.set_outputs([g.binary("add", g.unary("log", s), m)])
    return g


def scale_rows_cols(r, c):
    g = Graph()
    x, a, b = g.input(r, c), g.input(r, 1), g.input(1, c)
    g.set_outputs([g.binary("mul", g.binary("mul", x, g.bcast_colvec(a, c)), g.bcast_rowvec(b, r))])
    return g


def more_cases():
    """Patterns around the shape-modulation ops, masks and column statistics (`bench.py --survey` times them after `cases()`)."""
    out = []
    out.append(("dropout+residual bf16/u8", dropout_residual(16384, 4096), 16384, 4096))
    for r, c in [(65536, 256), (16384, 1024), (4096, 8192)]:
        out.append(("batchnorm f32", batchnorm(r, c), r, c))
    out.append(("softmax per 256-wide head bf16", heads_softmax(4096, 4096, 256), 4096, 4096))
    out.append(("softmax per 64-wide head bf16", heads_softmax(8192, 2048, 64), 8192, 2048))
    out.append(("concat+layernorm bf16", concat_layernorm(8192, 4096), 8192, 4096))
    out.append(("l2 normalise f32", l2_normalise(32768, 1024), 32768, 1024))
    out.append(("bias+transpose bf16", bias_transpose(8192, 4096), 8192, 4096))
    out.append(("gelu backward bf16", gelu_grad(16384, 4096), 16384, 4096))
    out.append(("logsumexp f32", logsumexp(8192, 32768), 8192, 32768))
    out.append(("logsumexp f32", logsumexp(65536, 1024), 65536, 1024))
    out.append(("scale rows and columns f32", scale_rows_cols(16384, 4096), 16384, 4096))
    # tensors of 4-16 MB: kernels of 4-25 us, where what happens after the last wavefront counts
    for r in (2048, 4096):
        out.append(("softmax f32", softmax_graph(r, 1024), r, 1024))
    out.append(("layernorm+gelu bf16", layernorm_gelu_graph(4096, 1024), 4096, 1024))
    out.append(("masked softmax bf16", masked_softmax(4096, 1024), 4096, 1024))
    out.append(("adam f32", adam(2048, 2048), 2048, 2048))
    return out


def cases():
    out = []
    for r, c in [(4096, 4096), (16384, 2048), (65536, 128), (8192, 8192), (2048, 32768), (1 << 20, 64), (4096, 65536), (2048, 131072)]:
        out.append(("softmax f32", softmax_graph(r, c), r, c))
    for r, c in [(32768, 768), (16384, 1024), (8192, 4096), (8192, 8192), (4096, 16384)]:
        out.append(("layernorm+gelu bf16", layernorm_gelu_graph(r, c), r, c))
        out.append(("rmsnorm bf16", rmsnorm(r, c), r, c))
    for r, c in [(16384, 1024), (8192, 4096)]:
        out.append(("add+layernorm bf16", add_layernorm(r, c), r, c))
        out.append(("masked softmax bf16", masked_softmax(r, c), r, c))
    for r, c in [(8192, 28672), (65536, 1024)]:
        out.append(("bias+gelu bf16", bias_gelu(r, c), r, c))
    for r, c in [(16384, 4096), (1, 1 << 26)]:
        out.append(("adam f32", adam(r, c), r, c))
    for r, c in [(1 << 20, 64), (65536, 1024), (16384, 4096), (1024, 65536)]:
        out.append(("column sum f32", colsum(r, c), r, c))
    out.append(("column sum bf16", colsum(65536, 1024, "bf16"), 65536, 1024))
    out.append(("bias grad f32", bias_grad(16384, 4096), 16384, 4096))
    for r, c in [(8192, 8192), (65536, 1024), (1024, 65536)]:
        out.append(("transpose f32", transpose(r, c), r, c))
    out.append(("transpose bf16", transpose(16384, 4096, "bf16"), 16384, 4096))
    for r, c in [(16384, 1024), (8192, 4096), (4096, 8192)]:
        out.append(("layernorm backward f32", layernorm_grad_graph(r, c), r, c))
    out.append(("softmax backward f32", softmax_grad_graph(8192, 4096), 8192, 4096))
    # a handful of very long rows: rows split over workgroups (norms), or cut into such kernels (softmax: 3 launches)
    for r, c in [(4, 1 << 22), (1, 1 << 26), (96, 1 << 19)]:
        out.append(("row L2 norm + max f32", row_norms(r, c), r, c))
    out.append(("softmax f32", softmax_graph(8, 1 << 20), 8, 1 << 20))
    # rows beyond one workgroup's registers: the head of the row stays in LDS between the stages
    out.append(("softmax f32", softmax_graph(2048, 100000), 2048, 100000))
    out.append(("layernorm+gelu bf16", layernorm_gelu_graph(4096, 65536), 4096, 65536))
    return out
