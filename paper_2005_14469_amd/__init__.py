"""fp32 sparse x dense multiplication (SpDM) with A in grouped-COO layout, for MI355X (gfx950).

The compute path lives in the HIP library under ``csrc/`` behind the C ABI
declared in ``include/gcoo.h``; ``binding`` marshals arguments to it.  The
library is loaded on first use and a missing build is a hard error: there is
no CPU fallback.
"""

__all__ = ["binding", "workloads"]
