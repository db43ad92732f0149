"""MI355X-native clustered-head decode attention (CHAI): Python face of the C-ABI library libchai.so.

The binding (and with it the shared library) is loaded on first use, so that `paper_2403_08058_amd.build` can be
imported to (re)build the library even when no library, or a stale one, is present.  There is no fallback: using
any entry point without a built library raises ImportError.
"""
import importlib

_BINDING_NAMES = ("CHAI_BF16", "CHAI_F32", "CHAI_OK", "EXPORTS", "LIB_PATH", "ChaiError", "alloc_workspace", "lib")


def __getattr__(name):
    if name == "build":
        return importlib.import_module(".build", __name__)
    binding = importlib.import_module(".binding", __name__)
    if name == "binding":
        return binding
    if name in _BINDING_NAMES or name in binding.EXPORTS:
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
