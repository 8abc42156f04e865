"""lpm: layer-wise partition-and-merge training step for one MI355X.

Thin Python binding over the C ABI declared in include/lpm.h.  Every arithmetic step runs in the
HIP library (liblpm.so); this package only marshals arguments and lays tensors out in device memory.
"""
from .binding import *          # noqa: F401,F403
from .binding import __all__    # noqa: F401
