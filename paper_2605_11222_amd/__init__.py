"""MI355X-native ADMM-Q layer solver: thin Python binding over the C-ABI library libadmmq.so.

Every step of the path runs inside the library's HIP kernels; this package only marshals arguments
(PyTorch tensors supply device memory and the stream).  Importing the package does not load the
library; the first call does, and fails loudly when it has not been built.
"""
from .binding import (  # noqa: F401
    AdmmqError,
    Context,
    Schedule,
    LayerStats,
    library_path,
    load_library,
    sample_pair,
    workspace_bytes,
    fast_products_bytes,
    EXPORTED_SYMBOLS,
    FORMAT_DUAL_GRID,
    FORMAT_CODEBOOK,
    NOALLOC_SCRATCH_BYTES,
)
