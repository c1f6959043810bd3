"""MI355X-native swap executor hot path (after SmartSwap, arXiv 2509.11076).

`paper_2509_11076_amd.binding` is the thin ctypes layer over libss.so (C ABI in
include/ss.h).  Names of the binding are reachable from the package directly
(`paper_2509_11076_amd.ss_swap_out`, ...); the library is loaded on first use
and its absence is an ImportError - there is no fallback path.
"""
import importlib

__all__ = ["binding", "build", "executor"]


def __getattr__(name):
    if name in ("binding", "build", "executor"):
        return importlib.import_module("." + name, __name__)
    b = importlib.import_module(".binding", __name__)
    try:
        return getattr(b, name)
    except AttributeError:
        raise AttributeError("module %r has no attribute %r" % (__name__, name)) from None
