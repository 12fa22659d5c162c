"""MI355X-native minibatch feature gather (GIDS, arxiv 2306.16384): thin
Python binding over the C ABI of libgids.so."""
from .binding import *  # noqa: F401,F403
from .binding import lib, LIB_PATH, EXPORTS, gids_stats, GidsError  # noqa: F401
