"""MI355X-native general binary tensor contraction  D := alpha*op(A)*op(B) + beta*op(C).

The product is the C-ABI library ``libtcx.so`` (declared in ``include/tcx.h``); this package is
its thin ctypes binding.  Every computation runs in the library's HIP kernels; the binding
only marshals arguments.  Importing :mod:`paper_2601_07827_amd.binding` fails loudly when the
library has not been built (``python paper_2601_07827_amd/build.py``).
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
