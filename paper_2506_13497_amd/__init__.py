"""libddit_hot for MI355X: the STDiT denoising step as HIP kernels behind a C ABI.

Importing the package loads the shared library; there is no CPU or PyTorch fallback."""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
