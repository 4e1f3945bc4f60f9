"""valvekv: preemptible paged-KV decode attention and KV reclamation on MI355X.

Thin ctypes binding over libvalvekv.so (C ABI declared in include/valvekv.h).
Every computation runs in the library's HIP kernels; this package only
marshals arguments.  There is no CPU fallback: the first use of any name of
the binding loads the built library and raises if it is missing.

(The binding is loaded on first attribute access so that
`python -m paper_2604_07874_amd.build` can run before the library exists.)
"""
import importlib

_binding = None


def _load_binding():
    global _binding
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    return _binding


def __getattr__(name):
    b = _load_binding()
    try:
        return getattr(b, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None


def __dir__():
    return sorted(set(globals()) | set(_load_binding().__all__))
