"""vt: attention over per-request, virtually contiguous KV caches on MI355X.

The package is a thin binding over libvt.so (C ABI in include/vt.h).  The binding is loaded on first
use so that `python -m paper_2407_15309_amd.build` can run before the library exists.
"""

import importlib

__all__ = ["binding"]


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    mod = importlib.import_module(".binding", __name__)
    if name == "binding":
        return mod
    try:
        return getattr(mod, name)
    except AttributeError:
        raise AttributeError("module %r has no attribute %r" % (__name__, name)) from None
