"""Layer-wise KV-cache load for MI355X: Python binding of libkvl.so (see include/kvl.h).

The binding (and with it the shared library) is loaded on first use, so that
``paper_2602_21548_amd.build`` can be imported and run while no library exists yet.
"""
import importlib

_EXPORTS = (
    "KvlError", "Plan", "make_layout", "kvl_plan", "kvl_pack_layer", "kvl_unpack_layer",
    "kvl_h2d_unpack_layer", "kvl_h2d_blockwise_layer", "kvl_stream_layers",
    "kvl_fullblocks_to_pool_layer", "kvl_h2d_fullblocks_layer", "kvl_d2h_pack_layer", "kvl_d2h_fullblocks_layer", "kvl_pool_to_fullblocks_layer", "kvl_plan_pair", "kvl_move_layer", "kvl_measure_h2d_peak", "kvl_copy_linear",
    "kvl_strerror", "kvl_release_cached_memory", "kvl_variant_name", "kvl_version", "LIB_PATH",
    "KVL_OK", "KVL_EINVAL", "KVL_ERANGE", "KVL_EALIAS", "KVL_ESPACE", "KVL_EHIP", "KVL_ENOMEM", "KVL_ENOSYS", "kvl_h2d_blockwise_batched_layer",
    "KVL_GATHER", "KVL_SCATTER", "KVL_HOST_ONLY", "KVL_NO_MERGE", "KVL_MAX_PLANES",
    "KVL_TOKENS_APPEND", "KVL_TOKENS_ALL", "KVL_NO_POINTER_CHECKS", "KVL_CALLER_SYNCS", "kvl_check_buffer",
    "kvl_unpack_layer_noalloc", "KVL_NOALLOC_MAX_UNITS",
    "kvl_ceiling_kernel", "KVL_CEILING_COPY", "KVL_CEILING_READ", "KVL_CEILING_WRITE",
)
__all__ = list(_EXPORTS)


def __getattr__(name):
    if name in _EXPORTS:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
