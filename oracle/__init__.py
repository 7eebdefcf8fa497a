"""CPU oracle of the W4A4 rotated linear layer (test infrastructure; see basq_oracle.py)."""
from .basq_oracle import *  # noqa: F401,F403
from . import basq_oracle as _impl

build = _impl.build
