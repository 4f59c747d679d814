"""MI355X-native hot path of REFT's in-memory checkpointing (arXiv 2310.12670) for one rank.

The product is ``libreft.so`` (hand-written HIP for gfx950 behind the C ABI of ``include/reft.h``);
this package is its thin Python binding: same names, argument marshalling only.  PyTorch supplies
device memory and streams, nothing else.  There is no CPU or PyTorch fallback: if the library is
not built, importing the binding's functions fails loudly.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
