"""MI355X-native paged multi-LoRA (Predictive-LoRA's page pool + shrink/expand kernels).

Thin ctypes binding over libplora.so (include/plora.h).  Importing this package loads the
library and fails loudly if it has not been built (python -m paper_2512_20210_amd.build):
there is no fallback path.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
