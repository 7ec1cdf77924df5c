"""MI355X-native DeltaKV hot path: residual compression and fused decode attention (gfx950 HIP).

The compute lives in libdeltakv.so (see include/deltakv.h); this package is the thin binding.
Importing it loads the library and raises ImportError if it has not been built.
"""
from . import binding  # noqa: F401  (loads libdeltakv.so or fails)
from .binding import (Dims, Layout, DeltaKVError, SPLIT, JOINT, METRIC_COSINE, METRIC_L2, make_dims,  # noqa: F401
                      paged_layout,
                      latent_block_offsets, keep_ratio, compress, decode_attn, version, strerror)
from .cache import PagedCache  # noqa: F401
