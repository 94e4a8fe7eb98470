"""FLuRKA attention (low-rank sequence projection + kernel feature map) for MI355X.

The compute lives in the C-ABI library built from `csrc/`; `binding` is the
thin ctypes layer over it and `inputs` draws the seeded synthetic workloads.
"""
from . import inputs  # noqa: F401
