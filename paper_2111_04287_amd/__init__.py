"""MI355X-native decentralized neighbor averaging (libbf) -- Python face of the C ABI.

The package is the shared library ``libbf.so`` (hand-written HIP for gfx950, built from
``csrc/``) plus ``binding``: ctypes wrappers carrying the C entry points' names.
"""

from .binding import *  # noqa: F401,F403
from .binding import lib, LIB_PATH, EXPORTS, BfError, Topology  # noqa: F401
