"""DynLP on AMD MI355X: dynamic batched label propagation behind a C-ABI HIP library.

``build()`` compiles ``csrc/dynlp.hip`` for gfx950 into ``libdynlp.so`` next to this file;
``DynLP`` (see ``binding``) is a thin ctypes wrapper with the same call names as the C ABI in
``include/dynlp.h``.  All computation happens in the HIP kernels; there is no CPU path, and
loading fails loudly if the library has not been built.
"""
from .build import build, library_path  # noqa: F401
from .binding import (DynLP, DynLPError, Stats, InitInfo, INIT_UNIFORM, INIT_SUPERNODE, UPDATE_SYNCHRONOUS, UPDATE_IN_PLACE,
                      load_library,  # noqa: F401
                      STATUS)
