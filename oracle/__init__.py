"""fp64 CPU oracle (test infrastructure).  See oracle.c for what it computes."""
from .oracle import *  # noqa: F401,F403
