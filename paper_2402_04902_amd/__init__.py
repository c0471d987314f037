"""MI355X-native L4Q layer (arXiv 2402.04902): HIP kernels behind a C ABI plus a thin binding.

`inputs` (seeded synthetic tensors) is importable anywhere.  `binding` loads libl4q.so on first
use and raises if the library has not been built; there is no CPU fallback.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "binding", "build"]
