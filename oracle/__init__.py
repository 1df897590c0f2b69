"""CPU oracle (test infrastructure only): see msx_oracle.c for what it defines."""
from .oracle import *  # noqa: F401,F403
