"""MI355X (gfx950) library for the per-block training step of Diversely Stale Parameters.

Everything is computed by hand-written HIP kernels behind the C ABI declared in
``include/dsp.h``; this package only loads the shared library and marshals arguments.
There is no CPU or PyTorch fallback: if the library is missing or no GPU is present the
calls fail loudly.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
