"""MI355X-native update-phase hot path of Deep Optimizer States (arXiv 2410.21316):
thin Python binding over libdos.so (HIP kernels + C ABI, see include/dos.h)."""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
