"""MI355X-native Fed-CVLC hot path (variable-length-code compression of
federated-learning model updates, arxiv 2402.03770).

`paper_2402_03770_amd.cvlc` is a thin binding over the C ABI declared in
include/cvlc.h: argument marshalling only, every step runs in libcvlc's HIP
kernels.  There is no CPU fallback: the binding raises if libcvlc.so has not
been built (python paper_2402_03770_amd/build.py).
"""
from . import cvlc  # noqa: F401
