"""libbnn for AMD MI355X: binarized FC / convolution layers on packed +1/-1 bits.

The compute path is the HIP library ``libbnn.so`` (see ``include/bnn.h``); this package is a thin
ctypes binding with the same names.  There is no CPU fallback: using any function without the
built library raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
