"""MI355X-native hot path of Chorus (three-stage inter-request caching for video
DiT serving): hand-written HIP kernels for gfx950 behind a C ABI (include/chorus.h)
and a ctypes binding with the same names. Importing the package does not load the
shared library; the first call does, and raises if it has not been built."""
from .binding import (ChorusError, chorus_cache_lookup, chorus_cache_lookup_batch, chorus_cache_lookup_static, chorus_denoise_schedule, chorus_dit_block_step,  # noqa: F401
                      chorus_dit_block_workspace_bytes, chorus_mask_hierarchy, chorus_mask_pooled_extent,
                      chorus_mask_project, chorus_region_blend, chorus_region_compact,
                      chorus_region_gather_rows, chorus_region_scatter_rows, load, lookup_result,
                      make_block_shape, upload_block_weights)
