"""MI355X-native conv-GLU + CTC training path (wav2letter++ acoustic-model hot path).

The product is ``libw2l.so`` (hand-written HIP for gfx950 behind a C ABI, see
``include/w2l.h``); this package is the thin binding that marshals torch device
tensors into it.  There is no CPU fallback: importing :mod:`binding` without the
built library raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib_path  # noqa: F401
