"""MI355X-native ADT pack / unpack and AWP layer statistics (arXiv 2004.02297).

Thin Python binding over the C-ABI library ``libadt.so`` (see include/adt.h).
PyTorch is used for device memory and streams only; every step of the method
on the weights runs in the library's gfx950 kernels.  There is no CPU fallback:
if the library is missing, loading fails.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    AWP_NSTATS, AdtError, AwpPlan, AwpState, adt_pack, adt_pack_unpack, adt_packed_size, adt_unpack16,
    adt_unpack,
    awp_layer_stats, awp_layer_stats_noalloc, awp_update, lib_path, load_library, adt_timing_enable,
    adt_timing_read, adt_stream_cache_limit, adt_launch_shape, awp_group_norms, awp_expand_group_bytes, adt_ablation, ABLATION_NAIVE, ABLATION_VEC_DIRECT, ABLATION_PER_LAYER,
)
