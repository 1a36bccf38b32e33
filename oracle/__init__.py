"""CPU oracle package (test infrastructure only; see sbp_oracle.py)."""
from .sbp_oracle import *  # noqa: F401,F403
from .sbp_oracle import build  # noqa: F401
