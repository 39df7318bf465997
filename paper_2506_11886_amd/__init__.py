"""MI355X-native FourierAttention hot path: `fa_compress`, `fa_decode`, `fa_append`, `fa_select_dims`.

A thin ctypes binding over the C ABI declared in include/fourier_attn.h.
Every step of the path runs in the HIP kernels of libfourier_attn.so; this
package only marshals torch tensors (device memory, streams) into pointers
and sizes.  There is no CPU fallback: a missing library is an ImportError.
"""

from .binding import (  # noqa: F401
    FA_OK, FA_ERR_NULL, FA_ERR_SHAPE, FA_ERR_UNSUPPORTED, FA_ERR_WORKSPACE, FA_ERR_HIP, FA_ERR_SCRATCH, FA_STATIC_SCRATCH_BYTES,
    FA_F32, FA_BF16, FA_KEEP_ROWS, FA_KEEP_TOK8,
    FA_MAX_HEAD_DIM, FA_MAX_GROUP, FA_MAX_STATES, FA_MAX_DECODE_STATES, FA_MAX_DECODE_STATES_F32, FA_MAX_KEPT_V_DIMS,
    FourierAttnError, lib, library_path, status_string,
    compress_workspace_bytes, decode_workspace_bytes, decode_default_splits,
    fa_compress, fa_compress_kv, compress_kv_workspace_bytes, fa_decode, fa_decode_varlen, fa_decode_static, fa_decode_mq, fa_append, fa_append_varlen, fa_select_dims, select_workspace_bytes, fa_legt, legt_workspace_bytes,
    keep_rows_from_tok8, tok8_numel, keep_rows_pitch,
)
