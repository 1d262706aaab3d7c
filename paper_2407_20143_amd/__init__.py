"""MI355X-native load-time checkpoint resharding (box-intersection planner + batched strided copy).

`binding` is the thin ctypes layer over the C-ABI library (include/bcp.h); `build` compiles the HIP
sources in-tree.  `synth` (seeded synthetic checkpoint layouts for the tests and the benchmark) is
not imported here: importing the package pulls in neither torch nor the generators.
"""
from . import binding  # noqa: F401
from .binding import (BcpError, Plan, configure, decompose, layout_to_meta,  # noqa: F401
                      meta_from_flat_slice, plan, reshard, validate_meta)
