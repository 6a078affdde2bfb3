"""Writes tests/golden/oracle_small_cases.json: outputs of the CPU oracle on tiny fixed inputs.

    python tests/golden/make_oracle_fixtures.py

Calls only `oracle/` and `workloads/` (never the GPU library).  The stored values serve two tests:
the oracle must keep reproducing them bit for bit (a guard against accidental changes to its
arithmetic), and the GPU path must match them within the usual tolerances.  Inputs are small
integers and dyadic fractions written out below, so a reader can redo a case by hand.
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from workloads import (bf16_bits_to_f32, f32_to_bf16_bits, layernorm_gelu_graph, layernorm_grad_graph, multi_reduce_graph,  # noqa: E402
                       softmax_graph, softmax_grad_graph)


def cases():
    x24 = np.array([[0.0, 1.0, 2.0, 3.0], [-1.0, -1.0, 0.5, 0.25]], dtype=np.float32)
    dy24 = np.array([[1.0, -2.0, 0.5, 0.0], [0.25, 0.0, -1.0, 4.0]], dtype=np.float32)
    ones4 = np.ones((1, 4), dtype=np.float32)
    return [
        ("softmax_2x4", softmax_graph(2, 4), [x24]),
        ("multi_reduce_2x4", multi_reduce_graph(2, 4), [x24]),
        ("layernorm_gelu_2x4_bf16", layernorm_gelu_graph(2, 4), [f32_to_bf16_bits(x24), ones4 * 1.5, ones4 * 0.25, ones4 * -0.125]),
        ("layernorm_grad_2x4", layernorm_grad_graph(2, 4), [x24, dy24, ones4 * 2.0]),
        ("softmax_grad_2x4", softmax_grad_graph(2, 4), [np.abs(x24) / 8.0, dy24]),
    ]


def main():
    out = {}
    for name, g, ins in cases():
        res = oracle.run(g, ins, 1)
        out[name] = {
            "inputs": [(bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64).tolist() for a in ins],
            "input_dtypes": ["bf16" if a.dtype == np.uint16 else "f32" for a in ins],
            # float32 / bf16 values as hex strings of their fp32 bit patterns: exact, diffable
            "outputs_hex": [[format(int(v), "08x") for v in
                             (bf16_bits_to_f32(r) if r.dtype == np.uint16 else r.astype(np.float32)).view(np.uint32).ravel()] for r in res],
            "output_shapes": [list(r.shape) for r in res],
        }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small_cases.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
    print("wrote", path)


if __name__ == "__main__":
    main()
