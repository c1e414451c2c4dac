"""CPU oracle (test infrastructure only; never imported by the product path).

The arithmetic lives in ``qnn_oracle.c``; this package compiles it with gcc and
exposes thin numpy wrappers.  Nothing here imports the HIP package.
"""
from .oracle import *  # noqa: F401,F403
