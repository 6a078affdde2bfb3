"""Comparison rule shared by the GPU parity tests.

Reference of record: the CPU oracle with every node rounded to its declared dtype ("A").

  u8 outputs    bit-exact.
  fp32 outputs  |gpu - A| <= rtol*|A| + rtol*rms(A), rtol = 1e-5.
  bf16 outputs  the same with rtol = 1e-2 (one bf16 ulp is 2^-8..2^-7 relative).

The rms term keeps the relative test meaningful at zeros and under cancellation below the
tensor's own scale.  Two refinements replace any blanket slack:

1. Quantisation decisions are shared (teacher forcing).  A COMPUTED bf16 node that other nodes
   consume is a quantiser: two correct implementations may round a value that sits on (or within
   an fp32 ulp of) the midpoint of two bf16 neighbours to either neighbour, and whatever is
   downstream inherits that 2^-8 relative step, amplified by cancellation, logarithms near 1, ...
   (three seeds of the random-graph sweep failed exactly so: an fp32 sigmoid/tanh result equal to
   a bf16 midpoint, rounded to even by the oracle, one fp32 ulp lower and hence rounded down on
   the device, followed by a subtraction of nearly equal values).  Such nodes must therefore be
   plan outputs of the graph under test (`expose_bf16_nodes`); the device's own bf16 values are
   checked against the oracle at the bf16 tolerance, and are then fed to the oracle IN PLACE of
   its own roundings, so that everything downstream is compared at its full tolerance with every
   rounding decision upstream being the device's.  bf16 INPUTS are exact on both sides.

2. Conditioning companions: the same oracle (B) with nodes kept in fp64 and rounded at plan
   outputs only, and (C) with every sum displaced by 2^-24 * sum |terms|, the first-order size of
   what accumulating in fp32 can do to a sum in any order.  The path under test rounds every node
   to fp32 and accumulates in fp32, in a tree order of its own; where A and B, or A and C, differ
   by more than the tolerance, the element is ill-conditioned with respect to exactly those choices
   (a row sum whose 5000 terms cancel to 0.1, behind a function that is steep at zero, is the case
   the random-graph sweep found), and no fp32 implementation can be held to the tolerance there.
   "More than the tolerance" is taken with a factor of four: the companions perturb by half an fp32
   ulp per node, the device's transcendental ops are good to 1-2 ulp (log(x) for x = 1.0019: one ulp
   of x is 1.2e-7 absolute in a tensor whose values are all ~1e-2 - another seed of the sweep).
   B and C each show ONE realisation of rounding noise, which at a given element can be small by chance (an fp32
   rounding that happened to be almost exact), while the device's own error there is not: a row maximum of differences
   of nearly equal tanh values - results ~5e-5 from operands ~1 - came out one operand spacing (6e-8, six tolerances)
   off at one element of one graph of the sweep with views, with |A - B| = 1e-9 there.  The third companion (S) is
   therefore not a realisation but the SCALE of the error: the oracle propagates, to first order, rounding noise
   (spacing/sqrt(12) per correctly rounded op and per partial sum of a pairwise summation; independent, added in
   quadrature) and the error of approximated ops (exp, log, tanh, sigmoid, rsqrt, rcp, gelu: 1-2 spacings on the
   device, one in the model; an approximation leans one way over a range of arguments, so these are added linearly -
   a row sum of 130 bounded terms was 1.01 tolerances off in another graph of that sweep) through every node.  An
   element whose spread S exceeds a quarter of its tolerance is flagged like the others.
   Those elements are counted and held to |gpu - A| <= 16*max(|A - B|, |A - C|) + 8*S + tol instead; a
   plan with more than a tenth of its output elements flagged fails as a test case (it would test
   little).  The random-graph generator squashes every reduction through tanh / sigmoid, so rows
   whose sums happen to cancel - a few per cent of the rows once a row has hundreds of terms - are
   flagged there; none is flagged in the benchmark workloads.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

import oracle
from workloads import Graph, bf16_bits_to_f32
from workloads.graph import Node

RTOL = {"f32": 1e-5, "bf16": 1e-2}
MAX_ILL_FRACTION = 0.1
ILL_SLACK = 16.0
# A companion moves a value by half an fp32 ulp per node (B) or one rounding unit per term (C); the device's
# transcendental ops are good to 1-2 ulp, i.e. up to four times B's perturbation.  An element is therefore flagged
# as soon as four times the companions' gap would exceed the tolerance.
ILL_THRESHOLD = 0.25
THREADS = 16


def _as_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    return (bf16_bits_to_f32(a) if dtype == "bf16" else a).astype(np.float64)


SPREAD_SLACK = 8.0


def check_output(gpu: np.ndarray, ref: np.ndarray, dtype: str, what: str = "", companions: Sequence[np.ndarray] = (),
                 spread: Optional[np.ndarray] = None):
    """One output tensor against reference A (and, when given, the conditioning companions B, C and the spread S).
    Returns statistics; "ill_conditioned" counts the elements the companions flagged (check_all bounds their share)."""
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    if dtype == "u8":
        bad = int((gpu != ref).sum())
        assert bad == 0, f"{what}: {bad} predicate bytes differ"
        return {"max_err_over_tol": 0.0, "ill_conditioned": 0}
    g, r = _as_f64(gpu, dtype), _as_f64(ref, dtype)
    assert np.isfinite(g).all(), f"{what}: non-finite GPU values"
    rtol = RTOL[dtype]
    s = float(np.sqrt(np.mean(r * r)))
    tol = rtol * np.abs(r) + rtol * s + 1e-37
    err = np.abs(g - r)
    n_ill = 0
    if len(companions) or spread is not None:
        gap = np.max([np.abs(_as_f64(c, dtype) - r) for c in companions], axis=0) if len(companions) else np.zeros_like(r)
        sd = spread if spread is not None else np.zeros_like(r)
        ill = (gap > ILL_THRESHOLD * tol) | (sd > ILL_THRESHOLD * tol)
        n_ill = int(ill.sum())
        if n_ill:
            tol = np.where(ill, ILL_SLACK * gap + SPREAD_SLACK * sd + tol, tol)
    ratio = float((err / tol).max())
    if ratio > 1.0:
        i = np.unravel_index(np.argmax(err / tol), err.shape)
        raise AssertionError(f"{what}: |gpu-ref|/tol = {ratio:.3g} at {i}: gpu {g[i]!r} ref {r[i]!r} (rms {s:.3g})")
    nrm = float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300))
    return {"max_err_over_tol": ratio, "normwise": nrm, "ill_conditioned": n_ill}


# ------------------------------------------------------------------------------------------------
# quantiser nodes
# ------------------------------------------------------------------------------------------------
# ops whose bf16 result is one of their bf16 operands' values (or its negation): no rounding decision is taken
_MOVES = ("reshape", "bitcast", "concat", "transpose", "bcast_rowvec", "bcast_colvec", "neg", "abs", "max", "min", "select")


def quantiser_nodes(graph: Graph) -> List[int]:
    """Computed bf16 nodes that round a value and that some other node consumes."""
    used = set()
    for n in graph.nodes:
        used.update(n.ins)

    def rounds(n):
        if n.dtype != "bf16" or n.op in ("input", "const"):
            return False
        values = n.ins[1:] if n.op == "select" else n.ins
        return not (n.op in _MOVES and all(graph.nodes[o].dtype == "bf16" for o in values))
    return [i for i, n in enumerate(graph.nodes) if rounds(n) and i in used]


def expose_bf16_nodes(graph: Graph) -> Graph:
    """The same DAG with every quantiser node added to the plan outputs (after the original ones)."""
    g = Graph(list(graph.nodes), list(graph.outputs))
    g.set_outputs(list(graph.outputs) + [q for q in quantiser_nodes(graph) if q not in graph.outputs])
    return g


def forced_graph(graph: Graph, forced: Sequence[int]):
    """The DAG in which every consumer of a node in `forced` reads a fresh bf16 INPUT instead.

    Returns (g2, computed, forced_input): computed[i] is the id in g2 of node i as the oracle
    computes it (from forced values upstream), forced_input[q] the id of the input standing in for q.
    """
    forced = set(forced)
    g2 = Graph()
    view, computed, forced_input = {}, {}, {}
    for i, n in enumerate(graph.nodes):
        c = g2._add(Node(n.op, n.dtype, n.rows, n.cols, tuple(view[o] for o in n.ins), n.attr, n.value, n.name))
        computed[i] = view[i] = c
        if i in forced:
            view[i] = forced_input[i] = g2.input(n.rows, n.cols, "bf16", name=f"forced_{i}")
    g2.set_outputs([computed[o] for o in graph.outputs])
    return g2, computed, forced_input


def _has_sums(graph: Graph) -> bool:
    return any(n.op in ("reduce_row", "reduce_col") and n.attr in ("sum", "mean") for n in graph.nodes)


class Reference:
    """Oracle results for one graph on one set of inputs: A, B, and per device run the forced forms."""

    def __init__(self, graph: Graph, inputs: Sequence[np.ndarray], threads: int = THREADS, with_b: bool = True):
        self.graph, self.inputs, self.threads, self.with_b = graph, list(inputs), threads, with_b
        self.quant = quantiser_nodes(graph)
        missing = [q for q in self.quant if q not in graph.outputs]
        assert not missing, (f"computed bf16 nodes {missing} are consumed inside the graph but are not plan outputs: "
                             "run the graph through expose_bf16_nodes() so their roundings can be shared")
        self._a = self._b = self._c = self._s = None

    @property
    def a(self) -> List[np.ndarray]:
        if self._a is None:
            self._a = oracle.run(self.graph, self.inputs, self.threads)
        return self._a

    @property
    def b(self) -> Optional[List[np.ndarray]]:
        if self._b is None and self.with_b:
            self._b = oracle.run(self.graph, self.inputs, self.threads, round_nodes=0)
        return self._b

    @property
    def c(self) -> Optional[List[np.ndarray]]:
        if self._c is None and self.with_b and _has_sums(self.graph):
            self._c = oracle.run(self.graph, self.inputs, self.threads, round_nodes=2)
        return self._c

    @property
    def s(self) -> Optional[List[np.ndarray]]:
        if self._s is None and self.with_b:
            self._s = oracle.run(self.graph, self.inputs, self.threads, round_nodes=3)
        return self._s

    def companions(self):
        return [x for x in (self.b, self.c) if x is not None]

    def __getitem__(self, k):
        return self.a[k]

    def __len__(self):
        return len(self.graph.outputs)

    def for_device(self, gpu_outs: Sequence[np.ndarray]):
        """(A, [companions], spreads) to compare `gpu_outs` with: the plain ones, or the forced ones when the graph has quantisers."""
        if not self.quant:
            return self.a, self.companions(), self.s
        g2, _, forced_input = forced_graph(self.graph, self.quant)
        by_new_id = {forced_input[q]: gpu_outs[self.graph.outputs.index(q)] for q in self.quant}
        originals = iter(self.inputs)
        ins2 = [by_new_id[i] if i in by_new_id else next(originals) for i in g2.input_ids()]
        a = oracle.run(g2, ins2, self.threads)
        modes = ([0] + ([2] if _has_sums(g2) else [])) if self.with_b else []
        return a, [oracle.run(g2, ins2, self.threads, round_nodes=m) for m in modes], (oracle.run(g2, ins2, self.threads, round_nodes=3) if self.with_b else None)


def check_all(graph: Graph, gpu_outs, ref, what: str = "", max_ill_fraction: float = MAX_ILL_FRACTION):
    """Every plan output of one device run against the oracle.  `ref` is a Reference (or a plain list of
    reference-A outputs for graphs without quantiser nodes: then there is no conditioning companion)."""
    if not isinstance(ref, Reference):
        assert not quantiser_nodes(graph), "a graph with consumed computed bf16 nodes needs a Reference"
        a, comps, spreads = list(ref), [], None
    else:
        a, comps, spreads = ref.for_device(gpu_outs)
    stats = []
    total = ill = 0
    for k, o in enumerate(graph.outputs):
        n = graph.nodes[o]
        stats.append(check_output(gpu_outs[k], a[k], n.dtype, f"{what} output {k} (node {o} {n.op} {n.name})", [c[k] for c in comps],
                                  spreads[k] if spreads is not None and n.dtype != "u8" else None))
        total += n.rows * n.cols
        ill += stats[-1]["ill_conditioned"]
    # (a floor of a few elements: a [4,1] output whose row sums cancel is two elements, not "half the workload")
    assert ill <= max(8.0, max_ill_fraction * total), \
        f"{what}: {ill} of {total} output elements are ill-conditioned (the oracle and its companions differ by more than the tolerance): the case tests nothing"
    return stats
