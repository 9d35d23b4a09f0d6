"""MI355X (gfx950) library for the hot path of the Orthrus dual-view decode step.

The product is ``liborthrus.so`` (hand-written HIP kernels behind the C ABI in
``include/orthrus.h``); this package is its build helper (``build``) and a ctypes binding with the
same entry-point names (``binding``, re-exported here).  The binding is loaded on first use of one of
its names, so that ``paper_2605_12825_amd.build`` can be imported to (re)build the library first.
"""
import importlib

_BINDING = None


def _binding():
    global _BINDING
    if _BINDING is None:
        _BINDING = importlib.import_module(__name__ + ".binding")
    return _BINDING


def __getattr__(name):
    if name in ("build", "binding", "runtime"):
        return importlib.import_module(__name__ + "." + name)
    b = _binding()
    try:
        return getattr(b, name)
    except AttributeError:
        raise AttributeError("module %r has no attribute %r" % (__name__, name)) from None
