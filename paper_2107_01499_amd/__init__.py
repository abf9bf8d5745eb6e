"""MI355X-native compression hot path of Bagua's communication primitives.

`from paper_2107_01499_amd import binding` loads lib/libbagua_hip.so (built by build.py); the
functions of `binding` carry the names of the C entry points declared in include/bagua_hip.h.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
