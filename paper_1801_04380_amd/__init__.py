"""MI355X (gfx950) kernels for the memory-budgeted CNN training step of
SuperNeurons (arXiv 1801.04380): convolution forward / backward with an explicit
workspace budget (Sec. 3.5), the planner that picks the fastest algorithm that
fits, and the cheap layers recomputation replays (Sec. 3.4).

This package is a thin binding over the C ABI in include/sn.h: every function
here only marshals arguments; all arithmetic runs in the HIP library.
"""
from .api import *  # noqa: F401,F403
from .api import __all__  # noqa: F401
