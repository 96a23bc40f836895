"""Single-MI355X kFkB pipeline-stage engine: thin Python binding over libkfkb.so.

All arithmetic runs in the HIP kernels behind the C boundary declared in include/kfkb.h;
this package only marshals arguments (PyTorch supplies device memory).  Importing it
does not load the library; the first call does, and fails loudly if it was not built.
"""
import os

from .binding import *          # noqa: F401,F403
from .binding import __all__    # noqa: F401
