"""CPU oracle for the Float8 linear hot path.  Test infrastructure only."""
from .f8_oracle import *  # noqa: F401,F403
