"""Thin Python binding over libdecoquant (C ABI declared in include/decoquant.h).

Argument marshalling only: every step of compression and decode attention runs in the HIP
kernels of the library.  torch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    DQError,
    Format,
    Cache,
    KVCacheLayer,
    ABI_VERSION,
    COMPRESS_NO_LARGE,
    COMPRESS_PLAIN,
    decode_flags,
    compress_flags,
    DECODE_AUTO,
    DECODE_FORCE_GENERIC,
    DECODE_FORCE_MFMA,
    EXPORTED_SYMBOLS,
    lib,
    version,
    status_string,
    alloc_cache,
    cache_from_numpy,
    decode_workspace,
    compress_workspace,
    workspace_init,
    attn_decode,
    compress_kv,
    compress_kv_blocks,
    cache_append,
    cache_append_workspace,
    APPEND_NO_COMPRESS,
    quantize_pack,
    stream_read,
    decode_mfma_supported,
)
