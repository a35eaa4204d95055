"""MI355X-native on-GPU decompression of the Endor bitmap sparse format.

`binding` is the thin ctypes layer over the C-ABI library (include/endor.h);
`synth` draws the seeded synthetic pruned matrices used as inputs.
"""
from . import binding, synth  # noqa: F401
from .binding import *  # noqa: F401,F403
