"""lpdt: MI355X-native hot path of low-precision decentralized training (arXiv 2111.09389).

Thin Python binding over the C-ABI library ``liblpdt.so`` (see ``include/lpdt.h``).
The binding only marshals arguments (torch tensors supply device memory and the
stream); every step of the path runs in the library's HIP kernels.  There is no
CPU fallback: importing works anywhere the library is built, calling needs a GPU.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
