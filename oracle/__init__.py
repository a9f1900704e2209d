"""CPU oracle (test infrastructure): see sage_oracle.py."""
from . import sage_oracle
from .sage_oracle import *  # noqa: F401,F403
