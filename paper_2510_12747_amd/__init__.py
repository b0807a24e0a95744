"""MI355X-native locality-constrained block-sparse attention (FlashVSR's self-attention hot path).

`binding` holds the ctypes wrappers of the C-ABI library (same names as include/lcsa.h);
`workloads` the benchmark shapes and the seeded synthetic inputs; `build` compiles the
HIP sources in-tree.  Importing the package does not load the shared library; the first
call through `binding` does, and raises if it has not been built.
"""
from .binding import (Cache, Geom, LcsaError, LCSA_BF16, LCSA_F32, WINDOW_PRESERVED, WINDOW_TRUNCATED,  # noqa: F401
                      lcsa_cache_device_bytes, lcsa_cache_frame_slot, lcsa_cache_init, lcsa_cache_pooled_k,
                      lcsa_cache_reset, lcsa_cache_valid_frames, lcsa_kv_cache_append, lcsa_pool_blocks,
                      lcsa_select_blocks, lcsa_sparse_attn_fwd, lcsa_status_string)
