"""MI355X (gfx950) implementation of BASE-Q's W4A4 rotated linear layer.

`binding` holds the ctypes wrappers of the C ABI declared in include/basq.h; `synth_inputs`
draws the seeded synthetic layers; `build` compiles libbasq.so with hipcc.  Nothing is loaded
at import time; the first binding call loads the library and raises if it is missing.
"""
from . import synth_inputs  # noqa: F401

__all__ = ["binding", "build", "synth_inputs"]
