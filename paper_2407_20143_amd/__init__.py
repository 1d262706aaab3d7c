"""MI355X-native load-time checkpoint resharding (box-intersection planner + batched strided copy).

`binding` is the thin ctypes layer over the C-ABI library (include/bcp.h); `synth` holds the
seeded synthetic checkpoint layouts used by the tests and the benchmark; `build` compiles the
HIP sources in-tree.
"""
from . import binding, synth  # noqa: F401
from .binding import (BcpError, Plan, configure, copy_baseline, decompose, layout_to_meta,  # noqa: F401
                      meta_from_flat_slice, plan, reshard)
