"""DEFT gradient-selection hot path for AMD MI355X: C-ABI library + thin binding."""
from . import synth  # noqa: F401
from . import binding  # noqa: F401  (loads libdeft.so lazily, on first call)
