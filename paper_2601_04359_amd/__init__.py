"""MI355X-native PackCache hot path: thin Python binding over libpackcache.so.

The HIP library is loaded on first use of a pc_* call and a missing library is an
error: there is no CPU fallback in this package.
"""
from .binding import *  # noqa: F401,F403
