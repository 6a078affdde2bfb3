"""Neutral description of a fusion plan: a DAG of named ops on 2-D tensors.

This module is shared by the CPU oracle's binding and the GPU library's binding.  It
holds no arithmetic of the method: only op *names*, shapes, dtypes and operand ids.
Each binding maps the names onto the enum values of its own C header.

The op vocabulary is the paper's problem statement (Section 2.1): elementwise ops,
shape modulation (broadcasts, transpose, reshape / bitcast; concat, Section 6.3) and reductions
(sum/max/min/mean, Section 1).  Tensors of any rank enter as [rows, cols] = [product of the leading
dims, product of the trailing dims] of their row-major layout; `reshape` moves that split.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

UNARY = ("neg", "abs", "exp", "log", "tanh", "sigmoid", "sqrt", "rsqrt", "rcp", "gelu_tanh", "convert")
BINARY = ("add", "sub", "mul", "div", "max", "min")
CMP_KINDS = ("gt", "ge", "lt", "le", "eq", "ne")
REDUCE_KINDS = ("sum", "max", "min", "mean")
DTYPES = ("f32", "bf16", "u8")
ALL_OPS = ("input", "const") + UNARY + BINARY + ("cmp", "select", "bcast_rowvec", "bcast_colvec",
                                                  "transpose", "reduce_row", "reduce_col", "reshape", "bitcast", "concat")
# nodes that are never materialised and never count as a kernel launch
FREE_OPS = ("input", "const", "bcast_rowvec", "bcast_colvec", "reshape", "bitcast")


@dataclass
class Node:
    op: str
    dtype: str
    rows: int
    cols: int
    ins: Tuple[int, ...] = ()
    attr: str = ""        # cmp kind / reduce kind
    value: float = 0.0    # const value
    name: str = ""


@dataclass
class Graph:
    nodes: List[Node] = field(default_factory=list)
    outputs: List[int] = field(default_factory=list)

    # ---- builders -------------------------------------------------------------
    def _add(self, node: Node) -> int:
        self.nodes.append(node)
        return len(self.nodes) - 1

    def shape(self, i: int) -> Tuple[int, int]:
        return self.nodes[i].rows, self.nodes[i].cols

    def input(self, rows: int, cols: int, dtype: str = "f32", name: str = "") -> int:
        return self._add(Node("input", dtype, rows, cols, (), name=name))

    def const(self, value: float, rows: int, cols: int, dtype: str = "f32") -> int:
        return self._add(Node("const", dtype, rows, cols, (), value=float(value)))

    def unary(self, op: str, a: int, dtype: str | None = None, name: str = "") -> int:
        assert op in UNARY, op
        n = self.nodes[a]
        return self._add(Node(op, dtype or n.dtype, n.rows, n.cols, (a,), name=name))

    def binary(self, op: str, a: int, b: int, dtype: str | None = None, name: str = "") -> int:
        assert op in BINARY, op
        n = self.nodes[a]
        return self._add(Node(op, dtype or n.dtype, n.rows, n.cols, (a, b), name=name))

    def cmp(self, kind: str, a: int, b: int, name: str = "") -> int:
        assert kind in CMP_KINDS, kind
        n = self.nodes[a]
        return self._add(Node("cmp", "u8", n.rows, n.cols, (a, b), attr=kind, name=name))

    def select(self, p: int, a: int, b: int, name: str = "") -> int:
        n = self.nodes[a]
        return self._add(Node("select", n.dtype, n.rows, n.cols, (p, a, b), name=name))

    def bcast_rowvec(self, v: int, rows: int) -> int:
        n = self.nodes[v]
        return self._add(Node("bcast_rowvec", n.dtype, rows, n.cols, (v,)))

    def bcast_colvec(self, v: int, cols: int) -> int:
        n = self.nodes[v]
        return self._add(Node("bcast_colvec", n.dtype, n.rows, cols, (v,)))

    def transpose(self, a: int, name: str = "") -> int:
        n = self.nodes[a]
        return self._add(Node("transpose", n.dtype, n.cols, n.rows, (a,), name=name))

    def reshape(self, a: int, rows: int, cols: int, name: str = "", op: str = "reshape") -> int:
        """The same row-major element sequence as [rows, cols] (op "bitcast": the same map under its other name)."""
        n = self.nodes[a]
        assert op in ("reshape", "bitcast") and rows * cols == n.rows * n.cols, (op, rows, cols, n.rows, n.cols)
        return self._add(Node(op, n.dtype, rows, cols, (a,), name=name))

    def view_nd(self, a: int, shape: Sequence[int], split: int, name: str = "") -> int:
        """Tensor `a` taken as an N-D tensor of `shape` and presented as [prod(shape[:split]), prod(shape[split:])]."""
        rows = 1
        for d in shape[:split]:
            rows *= d
        cols = 1
        for d in shape[split:]:
            cols *= d
        return self.reshape(a, rows, cols, name=name)

    def concat(self, a: int, b: int, axis: str = "cols", name: str = "") -> int:
        na, nb = self.nodes[a], self.nodes[b]
        assert axis in ("rows", "cols") and na.dtype == nb.dtype
        if axis == "cols":
            assert na.rows == nb.rows
            return self._add(Node("concat", na.dtype, na.rows, na.cols + nb.cols, (a, b), attr="cols", name=name))
        assert na.cols == nb.cols
        return self._add(Node("concat", na.dtype, na.rows + nb.rows, na.cols, (a, b), attr="rows", name=name))

    def reduce_row(self, kind: str, a: int, dtype: str | None = None, name: str = "") -> int:
        assert kind in REDUCE_KINDS, kind
        n = self.nodes[a]
        return self._add(Node("reduce_row", dtype or n.dtype, n.rows, 1, (a,), attr=kind, name=name))

    def reduce_col(self, kind: str, a: int, dtype: str | None = None, name: str = "") -> int:
        assert kind in REDUCE_KINDS, kind
        n = self.nodes[a]
        return self._add(Node("reduce_col", dtype or n.dtype, 1, n.cols, (a,), attr=kind, name=name))

    def set_outputs(self, ids: Sequence[int]) -> None:
        self.outputs = list(ids)

    # ---- queries ----------------------------------------------------------------
    def input_ids(self) -> List[int]:
        return [i for i, n in enumerate(self.nodes) if n.op == "input"]

    def compute_ids(self) -> List[int]:
        return [i for i, n in enumerate(self.nodes) if n.op not in FREE_OPS]

    def signature(self) -> str:
        """A stable text form (used for hashing a workload's DAG into reports)."""
        lines = []
        for i, n in enumerate(self.nodes):
            lines.append(f"{i}:{n.op}:{n.dtype}:{n.rows}x{n.cols}:{','.join(map(str, n.ins))}:{n.attr}:{n.value!r}")
        lines.append("out:" + ",".join(map(str, self.outputs)))
        return "\n".join(lines)


ELEM_BYTES = {"f32": 4, "bf16": 2, "u8": 1}


def min_hbm_bytes(g: Graph) -> int:
    """Bytes that must cross HBM at minimum: every plan input read once, every plan output written once."""
    total = 0
    for i in g.input_ids():
        n = g.nodes[i]
        total += n.rows * n.cols * ELEM_BYTES[n.dtype]
    for o in g.outputs:
        n = g.nodes[o]
        total += n.rows * n.cols * ELEM_BYTES[n.dtype]
    return total
