"""CPU oracle (test infrastructure only): see gids_oracle.c."""
from .oracle import *  # noqa: F401,F403
