"""CPU oracle of the stitched-kernel executor: TEST INFRASTRUCTURE ONLY.

Only tests, `__graft_entry__.smoke()` and `bench.py`'s cpu_baseline leg may import this
package.  It shares no code with the GPU library.
"""
from .binding import build, run, round_f32, round_bf16, lib_path  # noqa: F401
