"""MI355X-native expert-parallel dispatch/combine path (libep.so + ctypes binding)."""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
