"""MI355X-native per-GPU pipeline-stage forward (HexGen hot path).  See include/hexgen.h.

The ctypes binding (and with it libhexgen.so) is loaded on first use of any of its names, so that
`paper_2311_11514_amd.build` can be imported on a tree where the library has not been built yet.  There is no
fallback path: using the package without the built library raises ImportError."""
import importlib

_binding = None


def __getattr__(name):
    global _binding
    if name.startswith("__"):
        raise AttributeError(name)
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    try:
        return getattr(_binding, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None
