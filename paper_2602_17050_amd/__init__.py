"""MI355X-native MPZCH batched remap: thin Python binding over the C-ABI HIP library.

The binding (``paper_2602_17050_amd.binding``) is loaded lazily so that the
input generators in ``paper_2602_17050_amd.workloads`` can be imported on a
machine without the built library.
"""
import importlib

_BINDING_NAMES = (
    "load_library", "MpzchTable", "MpzchError",
    "mpzch_create", "mpzch_destroy", "mpzch_init_tensors", "mpzch_remap", "mpzch_lookup",
    "mpzch_reset_rows", "mpzch_remap_jagged", "mpzch_status_string",
    "mpzch_reset_rows_multi", "mpzch_lookup_gather", "mpzch_collect_delta", "mpzch_gather_rows", "mpzch_apply_delta",
    "EVICT_NONE", "EVICT_TTL", "EVICT_LRU", "EVICT_TTL_EXPIRY", "mpzch_remap_feature_ttl", "mpzch_remap_jagged_feature_ttl", "mpzch_lookup_jagged", "mpzch_reset_rows_jagged", "STAT_NAMES", "mpzch_create_with_layout", "mpzch_lookup_stats", "mpzch_remap_noalloc", "LAYOUT_SEPARATE", "LAYOUT_RECORDS",
)


def __getattr__(name):
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(__name__ + ".binding"), name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
