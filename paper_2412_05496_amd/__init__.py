"""FlexAttention hot path for AMD MI355X (gfx950): BlockMask builder, forward, backward and paged
decode as hand-written HIP kernels behind the C ABI of include/flexattn.h.

The Python layer only marshals arguments (see binding.py); importing the package does not load the
library, the first call does, and it raises if libflexattn.so has not been built.
"""
from .binding import *  # noqa: F401,F403
from .binding import (BlockMask, FlexAttnError, ModParams, alloc_blockmask, library_path)  # noqa: F401
