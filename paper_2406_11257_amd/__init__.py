"""MI355X-native ExCP checkpoint compression: thin Python binding of libexcp.so.

Every step of the method runs in the HIP library; this module only marshals
arguments (torch tensors -> device pointers) for the C ABI of include/excp.h.
There is no CPU fallback: loading fails loudly if the library is not built.
"""
from .binding import (  # noqa: F401
    EXCP_OK, EXCP_E_ARG, EXCP_E_CAP, EXCP_E_NONFINITE, EXCP_E_BLOB, EXCP_E_HIP, EXCP_E_STATE,
    EXCP_E_INTERNAL, EXCP_FLAG_MEDIAN_OF_WEIGHTS, EXCP_FLAG_NO_M2W, EXCP_FLAG_NO_QUANT, EXCP_FLAG_NO_W2M,
    EXCP_FLAG_W_F16, EXCP_FLAG_W_BF16, EXCP_PARAM_WIDE_ELEMS, EXCP_PARAM_CAND_LIST_ELEMS, ExcpError, ExcpStats, Context, PreparedBatch, lib, lib_path,
    excp_decompress_step_static, EXCP_STATIC_MAX_ELEMS, excp_blob_bound, excp_blob_size, excp_blob_size_ex, excp_dense_bytes, excp_head_bytes, excp_strerror,
)
