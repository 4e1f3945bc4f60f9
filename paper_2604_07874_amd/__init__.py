"""valvekv: preemptible paged-KV decode attention and KV reclamation on MI355X.

Thin ctypes binding over libvalvekv.so (C ABI declared in include/valvekv.h).
Every computation runs in the library's HIP kernels; this package only
marshals arguments.  There is no CPU fallback: importing `binding` without the
built library raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
