"""MI355X-native int4 compressed-domain decode attention (hand-written HIP behind a C ABI).

The Python layer only marshals arguments: every step of the path runs in the HIP kernels of
libtq_mi355x.so.  PyTorch is used for device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    KVCache,
    TqError,
    library_path,
    tq_decode_launches,
    tq_dense_scratch_bytes,
    tq_dequant_then_attend,
    tq_kv_bytes,
    tq_kv_bytes_grouped,
    tq_plan_splits,
    tq_quantize_kv,
    tq_quantize_kv_paged,
    tq_quantize_kv_varlen,
    tq_sdpa_int4_append_decode,
    tq_sdpa_int4_append_decode_paged,
    tq_sdpa_int4_append_decode_varlen,
    tq_sdpa_int4_decode,
    tq_sdpa_int4_decode_paged,
    tq_sdpa_int4_decode_static,
    tq_sdpa_int4_decode_varlen,
    tq_sdpa_int4_partial,
    tq_sdpa_int4_reduce,
    tq_status_string,
    tq_workspace_bytes,
    raw,
)
