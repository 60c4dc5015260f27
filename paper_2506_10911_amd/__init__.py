"""NoLoCo outer optimizer step for AMD MI355X (arxiv 2506.10911, Eq. 1-3).

The work is done by hand-written HIP kernels behind the C ABI of include/noloco.h; this
package is the thin Python binding to it (argument marshalling only).
"""
from .binding import (  # noqa: F401
    BF16, F32, LaunchPlan, NolocoError, copy_probe, library_path, merge_segments, outer_step,
    plan_groups, strerror,
)
