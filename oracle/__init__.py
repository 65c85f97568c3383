"""CPU fp64 oracle (test infrastructure only; never imported by the product path)."""
from .grid_code import *  # noqa: F401,F403
