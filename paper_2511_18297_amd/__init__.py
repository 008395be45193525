"""MI355X-native degree-split SpMM of GROOT (arXiv 2511.18297).

The package is a thin ctypes binding over ``libgroot.so`` (hand-written HIP for
gfx950 behind a C ABI, see ``include/groot.h``).  The binding is loaded on the
first use of any of its names, so that ``paper_2511_18297_amd.build`` can be
imported to compile the library in a tree that does not hold it yet; using the
package without the library raises ImportError (there is no fallback path).
"""
import importlib


def _binding():
    return importlib.import_module(".binding", __name__)


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    if name == "build":
        return importlib.import_module(".build", __name__)
    b = _binding()
    if name == "binding":
        return b
    try:
        return getattr(b, name)
    except AttributeError:
        raise AttributeError(f"module {__name__!r} has no attribute {name!r}") from None


def __dir__():
    return sorted(set(globals()) | set(dir(_binding())))
