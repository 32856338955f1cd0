"""Seeded synthetic inputs shared by the HIP path's callers and the oracle's callers."""
from .gen import *  # noqa: F401,F403
from .gen import __all__  # noqa: F401
