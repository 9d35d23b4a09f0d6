"""MI355X (gfx950) library for the hot path of the Orthrus dual-view decode step.

The product is ``liborthrus.so`` (hand-written HIP kernels behind the C ABI in
``include/orthrus.h``); this package is its build helper and a ctypes binding with the same
entry-point names.
"""
from .binding import *  # noqa: F401,F403
from .binding import (OrthrusError, make_params, orthrus_params, library_path, EXPORTED)  # noqa: F401
