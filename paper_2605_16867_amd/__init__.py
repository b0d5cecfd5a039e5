"""libgoodroute for MI355X: the batched routing math of GoodServe (Eq. 2,
Alg. 1, Sec. 3.4) as hand-written HIP kernels behind a C interface.

``binding`` wraps the shared library (loaded on first use, no fallback);
``workloads`` generates the seeded synthetic fleets; ``build`` compiles the
library with hipcc.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads", "binding", "build"]
