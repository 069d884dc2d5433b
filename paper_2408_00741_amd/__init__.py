"""MI355X-native batched evaluator of DynamoLLM's reconfiguration search space.

The work is done by hand-written HIP kernels in libdyn.so (C ABI: include/dyn.h);
`binding` marshals arguments to it.  There is no CPU fallback: importing `binding`
raises if the library has not been built (python paper_2408_00741_amd/build.py).
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
