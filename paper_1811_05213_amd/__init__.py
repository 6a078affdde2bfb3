"""Stitched execution of fused memory-bound tensor-op subgraphs on AMD MI355X (gfx950).

`binding` is the thin ctypes layer over the C-ABI library libfs.so (include/fs.h);
`runner` adds torch device-memory plumbing for tests and the benchmark.
"""
from .binding import (Plan, FsError, copy_probe, copy_probe_shape, launch_probe, alu_probe, device_limits, lib, FS_MODE_STITCHED, FS_MODE_UNFUSED, FS_MODE_NO_PERFLIB, FS_MODE_LAYERED, LIB_PATH)  # noqa: F401
