"""MI355X-native nano-batch decoder-layer forward: Python face of libdynlayer.so."""
from .binding import *  # noqa: F401,F403
