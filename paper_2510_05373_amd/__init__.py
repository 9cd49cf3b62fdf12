"""KVLinC 2-bit KV-cache decode path for AMD MI355X: thin Python binding over libkvlinc.so (C ABI, include/kvlinc.h).

Every step of the path runs in the HIP kernels of the library; this package only marshals arguments
(PyTorch supplies device memory and streams).  There is no CPU or PyTorch fallback: importing the
binding without the built library raises.
"""
from .binding import (  # noqa: F401
    KVLINC_EHIP, KVLINC_EINVAL, KVLINC_FLAG_ALG1_LITERAL, KVLINC_FLAG_SLIDING_VALUES, KVLINC_ESCRATCH, KVLINC_EWORKSPACE, KVLINC_OK, KVLINC_STATIC_SCRATCH_BYTES, KVLINC_ST_CAPACITY, KVLINC_ST_NONFINITE,
    KVLINC_ST_STATE_RANGE, KVLINC_ST_STATIC, CacheStruct, KVLincCache, KVLincError, kvlinc_append_quantize, kvlinc_cache_validate,
    kvlinc_decode_attention, kvlinc_decode_attention_noalloc, kvlinc_decode_attention_timed, kvlinc_decode_workspace_bytes, kvlinc_strerror, kvlinc_version, lib, lib_path,
)
