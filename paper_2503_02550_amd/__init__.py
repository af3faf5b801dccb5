"""MI355X-native SpecInF hot path: thin ctypes binding over libspecinf.so (see include/specinf.h)."""
from .binding import *  # noqa: F401,F403
