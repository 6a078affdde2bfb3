"""ctypes binding of the CPU oracle (oracle/fso.c).  Test infrastructure only."""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fso.c")
_LIB = os.path.join(_HERE, "libfso.so")

# op names -> enum values of fso.h (this binding's own table)
_OPC = {
    "input": 0, "const": 1, "neg": 2, "abs": 3, "exp": 4, "log": 5, "tanh": 6, "sigmoid": 7, "sqrt": 8,
    "rsqrt": 9, "rcp": 10, "gelu_tanh": 11, "convert": 12, "add": 13, "sub": 14, "mul": 15, "div": 16,
    "max": 17, "min": 18, "cmp": 19, "select": 20, "bcast_rowvec": 21, "bcast_colvec": 22, "transpose": 23,
    "reduce_row": 24, "reduce_col": 25, "reshape": 26, "bitcast": 27, "concat": 28,
}
_DT = {"f32": 0, "bf16": 1, "u8": 2}
_NP = {"f32": np.float32, "bf16": np.uint16, "u8": np.uint8}
_CMP = {"gt": 0, "ge": 1, "lt": 2, "le": 3, "eq": 4, "ne": 5}
_RED = {"sum": 0, "max": 1, "min": 2, "mean": 3}
_AXIS = {"rows": 0, "cols": 1}


class _Node(ctypes.Structure):
    _fields_ = [("opcode", ctypes.c_int32), ("dtype", ctypes.c_int32), ("rows", ctypes.c_int32),
                ("cols", ctypes.c_int32), ("num_in", ctypes.c_int32), ("inp", ctypes.c_int32 * 3),
                ("attr_i", ctypes.c_int32), ("attr_f", ctypes.c_float)]


class _Graph(ctypes.Structure):
    _fields_ = [("num_nodes", ctypes.c_int32), ("nodes", ctypes.POINTER(_Node)),
                ("num_outputs", ctypes.c_int32), ("outputs", ctypes.POINTER(ctypes.c_int32))]


def lib_path() -> str:
    return _LIB


def build(force: bool = False) -> str:
    """Compile oracle/fso.c with gcc into oracle/libfso.so (rebuilds when the source is newer)."""
    hdr = os.path.join(_HERE, "fso.h")
    stale = (not os.path.exists(_LIB)) or any(os.path.getmtime(p) > os.path.getmtime(_LIB) for p in (_SRC, hdr))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-Wall",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.fso_run.restype = ctypes.c_int
        _lib.fso_run.argtypes = [ctypes.POINTER(_Graph), ctypes.POINTER(ctypes.c_void_p),
                                 ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int]
        _lib.fso_round_f32.restype = ctypes.c_double
        _lib.fso_round_f32.argtypes = [ctypes.c_double]
        _lib.fso_round_bf16.restype = ctypes.c_double
        _lib.fso_round_bf16.argtypes = [ctypes.c_double]
    return _lib


def round_f32(x: float) -> float:
    return _load().fso_round_f32(float(x))


def round_bf16(x: float) -> float:
    return _load().fso_round_bf16(float(x))


def _encode(graph):
    n = len(graph.nodes)
    nodes = (_Node * n)()
    for i, nd in enumerate(graph.nodes):
        c = nodes[i]
        c.opcode = _OPC[nd.op]
        c.dtype = _DT[nd.dtype]
        c.rows, c.cols = nd.rows, nd.cols
        c.num_in = len(nd.ins)
        for k, o in enumerate(nd.ins):
            c.inp[k] = o
        c.attr_i = _CMP[nd.attr] if nd.op == "cmp" else _RED[nd.attr] if nd.op.startswith("reduce") else _AXIS[nd.attr] if nd.op == "concat" else 0
        c.attr_f = nd.value
    outs = (ctypes.c_int32 * max(1, len(graph.outputs)))(*graph.outputs)
    g = _Graph(n, nodes, len(graph.outputs), outs)
    return g, nodes, outs


def run(graph, inputs: Sequence[np.ndarray], num_threads: int = 1, round_nodes=True) -> List[np.ndarray]:
    """Evaluate `graph` (a workloads.Graph) on host arrays; returns one array per plan output.

    f32 tensors are float32 arrays, bf16 tensors are uint16 arrays of raw bits, u8 are uint8.
    round_nodes: True / 1 the reference of record; False / 0 the fp64 companion; 2 the fp32-accumulation companion;
    3 returns no values but float64 arrays of the first-order spread of a correct fp32 implementation around the reference.
    """
    lib = _load()
    g, _nodes, _outs = _encode(graph)
    in_ids = graph.input_ids()
    if len(inputs) != len(in_ids):
        raise ValueError(f"expected {len(in_ids)} inputs, got {len(inputs)}")
    held = []
    for i, arr in zip(in_ids, inputs):
        nd = graph.nodes[i]
        a = np.ascontiguousarray(arr, dtype=_NP[nd.dtype])
        if a.size != nd.rows * nd.cols:
            raise ValueError(f"input node {i}: expected {nd.rows}x{nd.cols}, got {arr.shape}")
        held.append(a)
    in_ptrs = (ctypes.c_void_p * max(1, len(held)))(*[a.ctypes.data for a in held])
    results = []
    for o in graph.outputs:
        nd = graph.nodes[o]
        results.append(np.empty((nd.rows, nd.cols), dtype=np.float64 if int(round_nodes) == 3 else _NP[nd.dtype]))
    out_ptrs = (ctypes.c_void_p * max(1, len(results)))(*[a.ctypes.data for a in results])
    rc = lib.fso_run(ctypes.byref(g), in_ptrs, out_ptrs, int(num_threads), int(round_nodes))
    if rc != 0:
        raise RuntimeError(f"fso_run failed with code {rc}")
    return results
