"""MI355X-native PipeMare training step: thin ctypes binding over libpipemare.so (HIP, gfx950)."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
