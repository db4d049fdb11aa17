"""MI355X (gfx950) u8 x s8 -> s32 GEMM: thin ctypes binding over the C-ABI HIP library.

The binding (and with it the shared library) is loaded on first use of any of its names, so
that `paper_1910_00178_amd.build` can (re)compile the library without loading a stale one.
There is no fallback: a missing or unloadable library raises.
"""
import importlib

_binding = None


def _load():
    global _binding
    if _binding is None:
        _binding = importlib.import_module(".binding", __name__)
    return _binding


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    if name in ("build", "workloads", "binding"):
        return importlib.import_module("." + name, __name__)
    return getattr(_load(), name)


def __dir__():
    return sorted(set(globals()) | set(dir(_load())))
