"""MI355X-native hot path of TCA-Attention behind a C ABI (libtca.so).

`binding` mirrors include/tca.h one to one; `buffers` allocates device memory
through torch.  Importing the package requires the built library.
"""
from . import binding  # noqa: F401  (raises ImportError if libtca.so is missing)
from .binding import *  # noqa: F401,F403
