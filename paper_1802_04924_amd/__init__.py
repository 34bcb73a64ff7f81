"""Layer-wise-parallelism strategy search (arXiv 1802.04924, Sec. 5) for one AMD MI355X.

`binding` is the ctypes face of the C ABI declared in include/lwp.h; `workloads` draws the
seeded synthetic inputs; `build` compiles the HIP sources.  Importing the package loads nothing:
the shared library is opened on first use and must have been built.
"""
from . import workloads  # noqa: F401
from .binding import (Context, LwpError, SCHEDULE_LEFT_FOLD, SCHEDULE_NONE, SCHEDULE_ROUNDS, UNDO_RECOMPUTE,  # noqa: F401
                      UNDO_STORED, enumerate_configs, plan_graph, search_workspace_bytes,
                      search_workspace_bytes_ragged)
