"""DiffQKV attention over an asymmetric KV cache for AMD MI355X (gfx950).

The product is ``libdiffqkv.so`` (hand-written HIP kernels behind the C ABI in ``include/diffqkv.h``);
this package is its thin Python binding plus the seeded input generators used by tests and benches.
"""
from . import inputs  # noqa: F401
from .binding import (  # noqa: F401
    BF16,
    F32,
    DiffQKVError,
    diffqkv_append,
    diffqkv_append_paged,
    diffqkv_decode,
    diffqkv_decode_paged,
    diffqkv_decode_static,
    diffqkv_decode_topk,
    diffqkv_decode_topk_paged,
    diffqkv_decode_workspace_bytes,
    diffqkv_prefill,
    diffqkv_probe_stream_read,
    diffqkv_kernel_timer,
    diffqkv_kernel_timer_read,
    diffqkv_set_tuning,
    diffqkv_version,
    load_library,
)
