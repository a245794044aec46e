"""FastH (arXiv 2009.13977) for AMD MI355X: HIP kernels behind a C ABI plus a thin ctypes binding.

`binding` exposes the entry points of include/fasth.h; `synthetic` draws the seeded test inputs;
`build` compiles the shared library with hipcc.
"""
from . import binding, synthetic  # noqa: F401
