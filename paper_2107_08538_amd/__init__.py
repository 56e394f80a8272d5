"""MI355X one-GPU task co-execution: thin ctypes binding over libmgb.so.

Argument marshalling only; every step (probe arithmetic, admission, CU
partitioning, kernels) runs inside the native library.  Importing this package
fails loudly if the library has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
