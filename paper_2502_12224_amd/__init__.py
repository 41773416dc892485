"""libfate: MI355X-native hot path of Fate's offloaded MoE inference.

The product is the C-ABI library built from csrc/ (see include/fate.h);
`binding` is its thin ctypes face.  Nothing here imports the CPU oracle.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
