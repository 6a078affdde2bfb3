"""ctypes binding of libfs.so: argument marshalling only, same names as include/fs.h.

Every step of the hot path runs inside the library's GPU kernels; this module converts a
`workloads.Graph` into the C structs and passes raw device pointers.  There is no CPU
fallback: if the library is missing the import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfs.so")

FS_ABI_VERSION = 2
FS_MODE_STITCHED = 0
FS_MODE_UNFUSED = 1
FS_MODE_NO_PERFLIB = 2
FS_MODE_LAYERED = 4
FS_STATIC_SCRATCH_BYTES = 8 << 20

STATUS_NAMES = ["FS_OK", "FS_ERR_INVALID_ARG", "FS_ERR_BAD_GRAPH", "FS_ERR_SHAPE", "FS_ERR_DTYPE", "FS_ERR_UNSUPPORTED",
                "FS_ERR_LDS_BUDGET", "FS_ERR_WORKSPACE", "FS_ERR_COMPILE", "FS_ERR_HIP", "FS_ERR_OOM"]

# op names -> fs_opcode values of include/fs.h (this binding's own table)
OPCODE = {
    "input": 0, "const": 1, "neg": 2, "abs": 3, "exp": 4, "log": 5, "tanh": 6, "sigmoid": 7, "sqrt": 8,
    "rsqrt": 9, "rcp": 10, "gelu_tanh": 11, "convert": 12, "add": 13, "sub": 14, "mul": 15, "div": 16,
    "max": 17, "min": 18, "cmp": 19, "select": 20, "bcast_rowvec": 21, "bcast_colvec": 22, "transpose": 23,
    "reduce_row": 24, "reduce_col": 25, "reshape": 26, "bitcast": 27, "concat": 28,
}
DTYPE = {"f32": 0, "bf16": 1, "u8": 2}
CMP = {"gt": 0, "ge": 1, "lt": 2, "le": 3, "eq": 4, "ne": 5}
RED = {"sum": 0, "max": 1, "min": 2, "mean": 3}
AXIS = {"rows": 0, "cols": 1}


class fs_node(ctypes.Structure):
    _fields_ = [("opcode", ctypes.c_int32), ("dtype", ctypes.c_int32), ("rows", ctypes.c_int32),
                ("cols", ctypes.c_int32), ("num_in", ctypes.c_int32), ("inp", ctypes.c_int32 * 3),
                ("attr_i", ctypes.c_int32), ("attr_f", ctypes.c_float)]


class fs_sched_hint(ctypes.Structure):
    _fields_ = [("lanes_per_row", ctypes.c_int32), ("wg_threads", ctypes.c_int32),
                ("max_workgroups", ctypes.c_int32), ("tiles_per_trip", ctypes.c_int32)]


class fs_graph_desc(ctypes.Structure):
    _fields_ = [("abi_version", ctypes.c_uint32), ("num_nodes", ctypes.c_int32), ("nodes", ctypes.POINTER(fs_node)),
                ("num_outputs", ctypes.c_int32), ("outputs", ctypes.POINTER(ctypes.c_int32)),
                ("group_of_node", ctypes.POINTER(ctypes.c_int32)), ("mode", ctypes.c_uint32),
                ("lds_budget_bytes", ctypes.c_int32), ("hint", ctypes.POINTER(fs_sched_hint))]


class fs_group_info(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("num_nodes", "dom_rows", "dom_cols", "lanes_per_row", "vec_elems", "elems_per_lane", "wg_threads",
                 "rows_per_iter", "grid", "lds_bytes", "num_row_reduces", "num_col_reduces", "num_ext_inputs",
                 "num_ext_outputs")] + [("min_hbm_bytes", ctypes.c_uint64), ("scratch_bytes", ctypes.c_uint64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class fs_tune_report(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("groups", "candidates", "measured", "hits", "improvable", "reserved")] + \
               [("current_usec", ctypes.c_double), ("best_usec", ctypes.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_ if n != "reserved"}


class FsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {message}")
        self.status = status
        self.status_name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libfs.so (built by `python -m paper_1811_05213_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_1811_05213_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p, u64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint64)
        L.fs_plan_create.argtypes = [ctypes.POINTER(fs_graph_desc), ctypes.POINTER(vp)]
        L.fs_plan_destroy.argtypes = [vp]
        L.fs_plan_workspace_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        L.fs_plan_run.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, ctypes.c_size_t, vp]
        L.fs_plan_workspace_init.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.fs_plan_stats.argtypes = [vp, i32p, i32p, u64p, u64p]
        L.fs_plan_group_info.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(fs_group_info)]
        L.fs_plan_node_groups.argtypes = [vp, i32p, ctypes.c_int32]
        L.fs_plan_node_spans.argtypes = [vp, i32p, ctypes.c_int32]
        L.fs_plan_group_source.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_char_p)]
        L.fs_plan_group_kernel_name.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_char_p)]
        L.fs_plan_group_perf_key.argtypes = [vp, ctypes.c_int32, ctypes.POINTER(ctypes.c_char_p)]
        L.fs_copy_probe.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.fs_plan_tune.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, ctypes.c_size_t, vp, ctypes.c_int32,
                                   ctypes.POINTER(fs_tune_report)]
        L.fs_plan_run_static.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp]
        L.fs_plan_run_static.restype = ctypes.c_int
        L.fs_copy_probe_shape.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32, vp]
        L.fs_copy_probe_shape.restype = ctypes.c_int
        L.fs_launch_probe.argtypes = [vp]
        L.fs_alu_probe.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp]
        L.fs_alu_probe.restype = ctypes.c_int
        L.fs_launch_probe.restype = ctypes.c_int
        L.fs_plan_load.argtypes = [vp]
        L.fs_plan_workspace_check.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.fs_plan_launched_hbm_bytes.argtypes = [vp, u64p]
        L.fs_device_limits.argtypes = [i32p, i32p, i32p, ctypes.POINTER(ctypes.c_int64), i32p]
        L.fs_last_error.restype = ctypes.c_char_p
        for name in ("fs_plan_create", "fs_plan_destroy", "fs_plan_workspace_bytes", "fs_plan_run",
                     "fs_plan_workspace_init", "fs_plan_stats", "fs_plan_group_info", "fs_plan_node_groups",
                     "fs_plan_group_source", "fs_plan_group_kernel_name", "fs_copy_probe", "fs_plan_tune", "fs_plan_group_perf_key", "fs_plan_node_spans",
                     "fs_plan_load", "fs_plan_workspace_check", "fs_plan_launched_hbm_bytes", "fs_device_limits"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise FsError(status, lib().fs_last_error().decode(errors="replace"))


def encode_graph(graph):
    """workloads.Graph -> (fs_node array, outputs array)."""
    n = len(graph.nodes)
    nodes = (fs_node * n)()
    for i, nd in enumerate(graph.nodes):
        c = nodes[i]
        c.opcode = OPCODE[nd.op]
        c.dtype = DTYPE[nd.dtype]
        c.rows, c.cols = nd.rows, nd.cols
        c.num_in = len(nd.ins)
        for k, o in enumerate(nd.ins):
            c.inp[k] = o
        c.attr_i = CMP[nd.attr] if nd.op == "cmp" else RED[nd.attr] if nd.op.startswith("reduce") else AXIS[nd.attr] if nd.op == "concat" else 0
        c.attr_f = nd.value
    outs = (ctypes.c_int32 * max(1, len(graph.outputs)))(*graph.outputs)
    return nodes, outs


class Plan:
    """Owns one fs_plan.  Methods mirror the C entry points one to one."""

    def __init__(self, graph, mode: int = FS_MODE_STITCHED, group_of_node: Optional[Sequence[int]] = None,
                 lds_budget_bytes: int = 0, hint: Optional[dict] = None):
        self.graph = graph
        nodes, outs = encode_graph(graph)
        desc = fs_graph_desc()
        desc.abi_version = FS_ABI_VERSION
        desc.num_nodes = len(graph.nodes)
        desc.nodes = nodes
        desc.num_outputs = len(graph.outputs)
        desc.outputs = outs
        grp = None
        if group_of_node is not None:
            grp = (ctypes.c_int32 * len(graph.nodes))(*group_of_node)
            desc.group_of_node = grp
        desc.mode = mode
        desc.lds_budget_bytes = lds_budget_bytes
        h = None
        if hint:
            h = fs_sched_hint(hint.get("lanes_per_row", 0), hint.get("wg_threads", 0), hint.get("max_workgroups", 0),
                              hint.get("tiles_per_trip", 0))
            desc.hint = ctypes.pointer(h)
        self._h = ctypes.c_void_p()
        self._run = lib().fs_plan_run
        _check(lib().fs_plan_create(ctypes.byref(desc), ctypes.byref(self._h)))

    def destroy(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().fs_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def workspace_bytes(self) -> int:
        n = ctypes.c_size_t()
        _check(lib().fs_plan_workspace_bytes(self._h, ctypes.byref(n)))
        return n.value

    def stats(self) -> dict:
        g, l = ctypes.c_int32(), ctypes.c_int32()
        a, b, c = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
        _check(lib().fs_plan_stats(self._h, ctypes.byref(g), ctypes.byref(l), ctypes.byref(a), ctypes.byref(b)))
        _check(lib().fs_plan_launched_hbm_bytes(self._h, ctypes.byref(c)))
        return {"num_groups": g.value, "num_launches": l.value, "min_hbm_bytes": a.value, "unfused_hbm_bytes": b.value,
                "launched_hbm_bytes": c.value}

    def run_static(self, input_ptrs: Sequence[int], output_ptrs: Sequence[int], stream: int = 0) -> None:
        ins, outs = self.pointer_tables(input_ptrs, output_ptrs)
        _check(lib().fs_plan_run_static(self._h, ins, outs, stream))

    def load(self) -> None:
        _check(lib().fs_plan_load(self._h))

    def workspace_check(self, workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> None:
        _check(lib().fs_plan_workspace_check(self._h, workspace_ptr, workspace_bytes, stream))

    def group_info(self, group: int) -> dict:
        info = fs_group_info()
        _check(lib().fs_plan_group_info(self._h, group, ctypes.byref(info)))
        return info.as_dict()

    def node_groups(self) -> List[int]:
        n = len(self.graph.nodes)
        out = (ctypes.c_int32 * n)()
        _check(lib().fs_plan_node_groups(self._h, out, n))
        return list(out)

    def node_spans(self) -> List[int]:
        n = len(self.graph.nodes)
        out = (ctypes.c_int32 * n)()
        _check(lib().fs_plan_node_spans(self._h, out, n))
        return list(out)

    def group_source(self, group: int) -> str:
        s = ctypes.c_char_p()
        _check(lib().fs_plan_group_source(self._h, group, ctypes.byref(s)))
        return s.value.decode()

    def group_kernel_name(self, group: int) -> str:
        s = ctypes.c_char_p()
        _check(lib().fs_plan_group_kernel_name(self._h, group, ctypes.byref(s)))
        return s.value.decode()

    def group_perf_key(self, group: int) -> str:
        s = ctypes.c_char_p()
        _check(lib().fs_plan_group_perf_key(self._h, group, ctypes.byref(s)))
        return s.value.decode()

    def workspace_init(self, workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> None:
        _check(lib().fs_plan_workspace_init(self._h, workspace_ptr, workspace_bytes, stream))

    def run(self, input_ptrs: Sequence[int], output_ptrs: Sequence[int], workspace_ptr: int, workspace_bytes: int,
            stream: int = 0) -> None:
        ins, outs = self.pointer_tables(input_ptrs, output_ptrs)
        _check(lib().fs_plan_run(self._h, ins, outs, workspace_ptr, workspace_bytes, stream))

    def tune(self, input_ptrs: Sequence[int], output_ptrs: Sequence[int], workspace_ptr: int, workspace_bytes: int,
             stream: int = 0, reps: int = 0) -> dict:
        ins, outs = self.pointer_tables(input_ptrs, output_ptrs)
        rep = fs_tune_report()
        _check(lib().fs_plan_tune(self._h, ins, outs, workspace_ptr, workspace_bytes, stream, reps, ctypes.byref(rep)))
        return rep.as_dict()

    @staticmethod
    def pointer_tables(input_ptrs: Sequence[int], output_ptrs: Sequence[int]):
        """The two host arrays of device pointers fs_plan_run takes (build once, reuse per launch)."""
        ins = (ctypes.c_void_p * max(1, len(input_ptrs)))(*input_ptrs)
        outs = (ctypes.c_void_p * max(1, len(output_ptrs)))(*output_ptrs)
        return ins, outs

    def run_tables(self, ins, outs, workspace_ptr: int, workspace_bytes: int, stream: int = 0) -> None:
        """fs_plan_run with pointer tables made by pointer_tables(): the cheapest call path from Python."""
        status = self._run(self._h, ins, outs, workspace_ptr, workspace_bytes, stream)
        if status != 0:
            _check(status)


def device_limits() -> dict:
    cu, lds, lanes, frm = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    l2 = ctypes.c_int64()
    _check(lib().fs_device_limits(ctypes.byref(cu), ctypes.byref(lds), ctypes.byref(lanes), ctypes.byref(l2), ctypes.byref(frm)))
    return {"compute_units": cu.value, "lds_bytes_per_workgroup": lds.value, "resident_lanes": lanes.value, "l2_bytes": l2.value,
            "from_device": bool(frm.value)}


def copy_probe_shape(src_ptr: int, dst_ptr: int, nbytes: int, vectors_in_flight: int, workgroups: int, stream: int = 0) -> None:
    _check(lib().fs_copy_probe_shape(src_ptr, dst_ptr, nbytes, vectors_in_flight, workgroups, stream))


def alu_probe(out_ptr: int, workgroups: int, iters: int, stream: int = 0) -> None:
    _check(lib().fs_alu_probe(out_ptr, workgroups, iters, stream))


def launch_probe(stream: int = 0) -> None:
    _check(lib().fs_launch_probe(stream))


def copy_probe(src_ptr: int, dst_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(lib().fs_copy_probe(src_ptr, dst_ptr, nbytes, stream))
