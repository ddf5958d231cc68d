"""MI355X-native Stream-K++ GEMM: thin Python face of libstreamk.so (see include/streamk.h)."""
from .binding import *  # noqa: F401,F403
from . import binding, inputs  # noqa: F401
