"""Comparison rule shared by the GPU parity tests.

fp32 outputs: |gpu - ref| <= rtol*|ref| + rtol*rms(ref) with rtol = 1e-5; bf16 outputs the same
with rtol = 1e-2; u8 outputs bit-exact.  The rms term keeps the relative test meaningful at
zeros and under cancellation (differences of nearly equal values, GeLU outputs near -0).
An fp32 output computed FROM a bf16-rounded intermediate is held to the bf16 tolerance: the two
sides may round that intermediate to neighbouring bf16 values (fp32 -> bf16 on the GPU, fp64 -> bf16
in the oracle, values one ulp apart across a rounding boundary), and everything downstream inherits
that relative 2^-8.  bf16 INPUTS are exact on both sides and do not count.
"""
import numpy as np

from workloads import bf16_bits_to_f32

RTOL = {"f32": 1e-5, "bf16": 1e-2}


def check_output(gpu: np.ndarray, ref: np.ndarray, dtype: str, what: str = "", rtol_scale: float = 1.0):
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    if dtype == "u8":
        bad = int((gpu != ref).sum())
        assert bad == 0, f"{what}: {bad} predicate bytes differ"
        return {"max_err_over_tol": 0.0}
    if dtype == "bf16":
        gpu, ref = bf16_bits_to_f32(gpu), bf16_bits_to_f32(ref)
    g = gpu.astype(np.float64)
    r = ref.astype(np.float64)
    assert np.isfinite(g).all(), f"{what}: non-finite GPU values"
    rtol = RTOL[dtype] * rtol_scale
    s = float(np.sqrt(np.mean(r * r)))
    tol = rtol * np.abs(r) + rtol * s + 1e-37
    err = np.abs(g - r)
    ratio = float((err / tol).max())
    if ratio > 1.0:
        i = np.unravel_index(np.argmax(err / tol), err.shape)
        raise AssertionError(f"{what}: |gpu-ref|/tol = {ratio:.3g} at {i}: gpu {g[i]!r} ref {r[i]!r} (rms {s:.3g})")
    nrm = float(np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-300))
    return {"max_err_over_tol": ratio, "normwise": nrm}


def through_bf16(graph):
    """For every node: does its value depend on a COMPUTED bf16 node?"""
    dep = [False] * len(graph.nodes)
    for i, n in enumerate(graph.nodes):
        dep[i] = (n.dtype == "bf16" and n.op != "input") or any(dep[o] for o in n.ins)
    return dep


def check_all(graph, gpu_outs, ref_outs, what="", rtol_scale: float = 1.0):
    stats = []
    dep = through_bf16(graph)
    for k, o in enumerate(graph.outputs):
        n = graph.nodes[o]
        scale = rtol_scale * (RTOL["bf16"] / RTOL["f32"] if n.dtype == "f32" and dep[o] else 1.0)
        stats.append(check_output(gpu_outs[k], ref_outs[k], n.dtype, f"{what} output {k} (node {o} {n.op} {n.name})", scale))
    return stats
