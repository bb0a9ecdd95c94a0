"""rslx: MI355X-native PPO / BC / symmetry / RND hot path.  Thin ctypes binding over librslx.so.

Every step runs in the HIP kernels of the shared library; this package only marshals arguments
(torch tensors provide device memory and the stream).  Importing the binding fails loudly when the
library has not been built (python paper_2509_10771_amd/build.py).
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
