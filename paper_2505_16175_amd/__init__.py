"""QuickPrefill hot path for MI355X: hand-written HIP kernels behind a C ABI (include/qp.h).

`binding` mirrors the C entry points one to one; `workload` makes the seeded synthetic inputs.
"""
from . import workload  # noqa: F401
from . import binding  # noqa: F401
