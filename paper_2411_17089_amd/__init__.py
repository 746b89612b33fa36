"""KVPR per-layer decode path for AMD MI355X: thin Python binding over libkvpr.so (HIP, gfx950)."""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, lib  # noqa: F401
