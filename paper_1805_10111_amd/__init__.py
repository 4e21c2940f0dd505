"""Double quantization (AsyLPG / Sparse-AsyLPG / Acc-AsyLPG) hot path on AMD MI355X.

Thin Python binding over ``libdq.so`` (hand-written HIP for gfx950, C ABI declared in
``include/dq.h``).  The binding only marshals arguments: every step of the method runs
in the library's kernels.  PyTorch supplies device memory and streams.  There is no
CPU fallback: importing :mod:`paper_1805_10111_amd.api` fails if the library has not
been built (``python paper_1805_10111_amd/build.py``).
"""
from .api import *  # noqa: F401,F403
from .api import __all__  # noqa: F401
