"""ctypes binding of libfourier_attn.so (argument marshalling only)."""

from __future__ import annotations

import ctypes
import os

import torch  # imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfourier_attn.so")

FA_OK = 0
FA_ERR_NULL, FA_ERR_SHAPE, FA_ERR_UNSUPPORTED, FA_ERR_WORKSPACE, FA_ERR_HIP, FA_ERR_SCRATCH = -1, -2, -3, -4, -5, -6
FA_STATIC_SCRATCH_BYTES = 8 << 20
FA_F32, FA_BF16 = 0, 1
FA_KEEP_ROWS, FA_KEEP_TOK8 = 0, 1
# compiled limits, as declared in include/fourier_attn.h
FA_MAX_HEAD_DIM = 256
FA_MAX_GROUP = 16
FA_MAX_STATES = 1024
FA_MAX_DECODE_STATES = 1024
FA_MAX_DECODE_STATES_F32 = 256
FA_MAX_KEPT_V_DIMS = 128


class FourierAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def library_path() -> str:
    return _LIB_PATH


def _load(path: str = _LIB_PATH):
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python paper_2506_11886_amd/build.py` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i32, i64, f32, sz = c.c_void_p, c.c_int, c.c_int64, c.c_float, c.c_size_t
    lib.fa_compress.restype = i32
    lib.fa_compress.argtypes = [vp, i32, i64, i64, i64, i32, i32, i32, i32, vp, i32,
                                i32, i32, i32, i32, vp, vp, i32, i64, i32, vp, sz, vp]
    lib.fa_compress_timed.restype = i32
    lib.fa_compress_timed.argtypes = lib.fa_compress.argtypes + [c.POINTER(c.c_float)]
    lib.fa_compress_workspace_bytes.restype = sz
    lib.fa_compress_workspace_bytes.argtypes = [i32] * 6
    lib.fa_compress_workspace_bytes_for.restype = sz
    lib.fa_compress_workspace_bytes_for.argtypes = [i32] * 7
    lib.fa_compress_kv_workspace_bytes_for.restype = sz
    lib.fa_compress_kv_workspace_bytes_for.argtypes = [i32] * 8
    lib.fa_decode.restype = i32
    lib.fa_decode.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, i32, vp, vp, i32,
                              i32, i32, i32, i32, vp, i64, vp, i64, vp, vp, i32, i64,
                              f32, i32, vp, vp, sz, vp]
    lib.fa_decode_timed.restype = i32
    lib.fa_decode_timed.argtypes = lib.fa_decode.argtypes + [c.POINTER(c.c_float)]
    lib.fa_decode_varlen.restype = i32
    lib.fa_decode_varlen.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, i32, vp, vp, i32,
                                     i32, i32, i32, i32, vp, vp, i64, vp, i64, vp, vp, i32, vp, i64,
                                     f32, i32, vp, vp, sz, vp]
    lib.fa_decode_static.restype = i32
    lib.fa_decode_static.argtypes = lib.fa_decode.argtypes[:27] + [vp]
    lib.fa_decode_workspace_bytes.restype = sz
    lib.fa_decode_workspace_bytes.argtypes = [i32] * 10
    lib.fa_decode_default_splits.restype = i32
    lib.fa_decode_default_splits.argtypes = [i32] * 6
    lib.fa_append.restype = i32
    lib.fa_append.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, i32, i64, i32, i32,
                              vp, i32, vp, i32, i32, i32, i32, vp, vp, vp, i64, vp, i64, vp]
    lib.fa_append_varlen.restype = i32
    lib.fa_append_varlen.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, i32, i64, vp,
                                     vp, i32, vp, i32, i32, i32, vp, i32, vp, vp, vp, i64, vp, i64, vp]
    lib.fa_compress_kv_workspace_bytes.restype = sz
    lib.fa_compress_kv_workspace_bytes.argtypes = [i32] * 7
    lib.fa_compress_kv.restype = i32
    lib.fa_compress_kv.argtypes = [vp, vp, i32, i64, i64, i64, i32, i32, i32, i32, vp, i32, vp, i32,
                                   i32, i32, i32, i32, vp, vp, vp, i64, vp, i64, i32, vp, sz, vp]
    lib.fa_compress_kv_timed.restype = i32
    lib.fa_compress_kv_timed.argtypes = lib.fa_compress_kv.argtypes + [c.POINTER(c.c_float)]
    lib.fa_decode_mq.restype = i32
    lib.fa_decode_mq.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, i32, vp, vp, i32,
                                 i32, i32, i32, i32, vp, i64, vp, i64, vp, vp, i32, i64,
                                 f32, i32, vp, vp, sz, vp]
    lib.fa_select_workspace_bytes.restype = sz
    lib.fa_select_workspace_bytes.argtypes = [i32] * 6
    lib.fa_select_dims.restype = i32
    lib.fa_select_dims.argtypes = [vp, i32, i64, i64, i64, i32, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.fa_legt_workspace_bytes.restype = sz
    lib.fa_legt_workspace_bytes.argtypes = [i32] * 5
    lib.fa_legt_compress.restype = i32
    lib.fa_legt_compress.argtypes = [vp, i32, i64, i64, i64, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.fa_legt_mse.restype = i32
    lib.fa_legt_mse.argtypes = [vp, i32, i64, i64, i64, i32, i32, i32, i32, i32, vp, vp, vp, sz, vp]
    lib.fa_status_string.restype = c.c_char_p
    lib.fa_status_string.argtypes = [i32]
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.fa_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FA_F32
    if t.dtype == torch.bfloat16:
        return FA_BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def compress_workspace_bytes(B, H, N, D, Dc, M, dtype=None) -> int:
    """Workspace of fa_compress: for one element type (a torch dtype or FA_* code) when given, else
    the figure that covers either."""
    if dtype is None:
        return int(lib.fa_compress_workspace_bytes(B, H, N, D, Dc, M))
    code = dtype if isinstance(dtype, int) else (FA_F32 if dtype == torch.float32 else FA_BF16)
    return int(lib.fa_compress_workspace_bytes_for(code, B, H, N, D, Dc, M))


def decode_workspace_bytes(B, Hq, Hkv, D, Dkc, Dvc, M, N, W, num_splits=0) -> int:
    return int(lib.fa_decode_workspace_bytes(B, Hq, Hkv, D, Dkc, Dvc, M, N, W, num_splits))


def decode_default_splits(B, Hq, Hkv, M, N, W) -> int:
    return int(lib.fa_decode_default_splits(B, Hq, Hkv, M, N, W))


def keep_rows_pitch(Du: int) -> int:
    """Row pitch (elements) of the FA_KEEP_ROWS layout: Du rounded up to 8."""
    return (Du + 7) // 8 * 8


def tok8_numel(n_tokens: int, Du: int) -> int:
    """Elements of one FA_KEEP_TOK8 slab holding n_tokens tokens of Du dims."""
    return (n_tokens + 7) // 8 * 8 * Du


def keep_rows_from_tok8(t: torch.Tensor, n_tokens: int, Du: int) -> torch.Tensor:
    """View helper for tests: [..., ceil(n/8), Du, 8] slab -> [..., n, Du] rows."""
    lead = t.shape[:-1]
    g = (n_tokens + 7) // 8
    x = t.reshape(*lead, g, Du, 8).transpose(-1, -2).reshape(*lead, g * 8, Du)
    return x[..., :n_tokens, :]


def fa_compress(x, dim_mask, Dc, M, T, t0=0, accumulate=False, coeffs=None, x_keep=None,
                keep_layout=FA_KEEP_ROWS, keep_offset=0, keep_stride_bh=0,
                workspace=None, stream=None, kernel_ms=None):
    """Enqueue fa_compress on `stream`.

    x [B,H,N,D] (last dim contiguous), dim_mask uint8 [B,H,D].  Allocates the
    outputs / workspace with torch when they are not passed.  Returns
    (coeffs [B,H,M,Dc] fp32, x_keep).  With `kernel_ms` (a list) the timed,
    synchronous entry point is used and the per-kernel milliseconds appended.
    """
    B, H, N, D = x.shape
    assert x.stride(3) == 1 or N == 0
    dev = x.device
    if coeffs is None:
        coeffs = torch.empty((B, H, M, Dc), dtype=torch.float32, device=dev)
    Du = D - Dc
    if x_keep is None:
        n_tok = keep_offset + N
        if keep_layout == FA_KEEP_ROWS:
            x_keep = torch.empty((B, H, n_tok, keep_rows_pitch(Du)), dtype=x.dtype, device=dev)
        else:
            x_keep = torch.zeros((B, H, tok8_numel(n_tok, Du)), dtype=x.dtype, device=dev)
    need = compress_workspace_bytes(B, H, N, D, Dc, M, x.dtype)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    args = (_ptr(x), _dtype_code(x), x.stride(0), x.stride(1), x.stride(2),
            B, H, N, D, _ptr(dim_mask), Dc, M, T, t0, int(bool(accumulate)),
            _ptr(coeffs), _ptr(x_keep), keep_layout, keep_stride_bh, keep_offset,
            _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if kernel_ms is None:
        st = lib.fa_compress(*args)
    else:
        ms = (ctypes.c_float * 2)()
        st = lib.fa_compress_timed(*args, ms)
        kernel_ms.extend(ms)
    if st != FA_OK:
        raise FourierAttnError(st, "fa_compress")
    return coeffs, x_keep


def fa_decode(q, ck, kmask, cv, vmask, M, T, t0, N, k_keep, v_keep, k_full, v_full,
              scale=0.0, num_splits=0, out=None, workspace=None, stream=None,
              kk_stride_bh=0, vk_stride_bh=0, full_stride_bh=0, kernel_ms=None):
    """Enqueue fa_decode on `stream`; returns out [B,Hq,D] fp32.  With
    `kernel_ms` (a list) the timed, synchronous entry point is used and the
    per-kernel milliseconds (prepare, partial, finish) appended."""
    B, Hq, D = q.shape
    Hkv = kmask.shape[1]
    Dkc = ck.shape[-1] if ck is not None else 0
    Dvc = cv.shape[-1] if cv is not None else 0
    W = k_full.shape[2] if k_full is not None else 0
    dev = q.device
    if out is None:
        out = torch.empty((B, Hq, D), dtype=torch.float32, device=dev)
    if workspace is None:
        need = decode_workspace_bytes(B, Hq, Hkv, D, Dkc, Dvc, M, N, W, num_splits)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    args = (_ptr(q), _dtype_code(q), B, Hq, Hkv, D,
            _ptr(ck), _ptr(kmask), Dkc, _ptr(cv), _ptr(vmask), Dvc,
            M, T, t0, N, _ptr(k_keep), kk_stride_bh, _ptr(v_keep), vk_stride_bh,
            _ptr(k_full), _ptr(v_full), W, full_stride_bh,
            float(scale), num_splits, _ptr(out),
            _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if kernel_ms is None:
        st = lib.fa_decode(*args)
    else:
        ms = (ctypes.c_float * 3)()
        st = lib.fa_decode_timed(*args, ms)
        kernel_ms.extend(ms)
    if st != FA_OK:
        raise FourierAttnError(st, "fa_decode")
    return out


def fa_decode_varlen(q, ck, kmask, cv, vmask, M, T, t0, N_max, seq_n, k_keep, v_keep, k_full, v_full, seq_w,
                     scale=0.0, num_splits=0, out=None, workspace=None, stream=None,
                     kk_stride_bh=0, vk_stride_bh=0, full_stride_bh=0):
    """Enqueue fa_decode_varlen: `seq_n` / `seq_w` are int32 device tensors [B] (or None) with each
    sequence's middle-row and full-width-row counts; everything else as fa_decode."""
    B, Hq, D = q.shape
    Hkv = kmask.shape[1]
    Dkc = ck.shape[-1] if ck is not None else 0
    Dvc = cv.shape[-1] if cv is not None else 0
    W = k_full.shape[2] if k_full is not None else 0
    dev = q.device
    for t in (seq_n, seq_w):
        if t is not None and (t.dtype != torch.int32 or t.numel() != B or not t.is_contiguous()):
            raise ValueError("seq_n / seq_w must be contiguous int32 tensors of B entries")
    if out is None:
        out = torch.empty((B, Hq, D), dtype=torch.float32, device=dev)
    if workspace is None:
        need = decode_workspace_bytes(B, Hq, Hkv, D, Dkc, Dvc, M, N_max, W, num_splits)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    st = lib.fa_decode_varlen(_ptr(q), _dtype_code(q), B, Hq, Hkv, D,
                              _ptr(ck), _ptr(kmask), Dkc, _ptr(cv), _ptr(vmask), Dvc,
                              M, T, t0, N_max, _ptr(seq_n), _ptr(k_keep), kk_stride_bh, _ptr(v_keep), vk_stride_bh,
                              _ptr(k_full), _ptr(v_full), W, _ptr(seq_w), full_stride_bh,
                              float(scale), num_splits, _ptr(out),
                              _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if st != FA_OK:
        raise FourierAttnError(st, "fa_decode_varlen")
    return out


def fa_decode_static(q, ck, kmask, cv, vmask, M, T, t0, N, k_keep, v_keep, k_full, v_full,
                     scale=0.0, num_splits=0, out=None, stream=None,
                     kk_stride_bh=0, vk_stride_bh=0, full_stride_bh=0):
    """Enqueue fa_decode_static on `stream`: fa_decode with the split-K state in the library's
    static device array (no workspace; the call itself allocates nothing when `out` is passed)."""
    B, Hq, D = q.shape
    Hkv = kmask.shape[1]
    Dkc = ck.shape[-1] if ck is not None else 0
    Dvc = cv.shape[-1] if cv is not None else 0
    W = k_full.shape[2] if k_full is not None else 0
    if out is None:
        out = torch.empty((B, Hq, D), dtype=torch.float32, device=q.device)
    st = lib.fa_decode_static(_ptr(q), _dtype_code(q), B, Hq, Hkv, D,
                              _ptr(ck), _ptr(kmask), Dkc, _ptr(cv), _ptr(vmask), Dvc,
                              M, T, t0, N, _ptr(k_keep), kk_stride_bh, _ptr(v_keep), vk_stride_bh,
                              _ptr(k_full), _ptr(v_full), W, full_stride_bh,
                              float(scale), num_splits, _ptr(out), _stream_ptr(stream))
    if st != FA_OK:
        raise FourierAttnError(st, "fa_decode_static")
    return out


def fa_append(k_new, v_new, k_full, v_full, slot, evict, kmask=None, vmask=None, M=0, T=0, n_mid=0,
              ck=None, cv=None, k_keep=None, v_keep=None, stream=None,
              kk_stride_bh=0, vk_stride_bh=0, full_stride_bh=0):
    """Enqueue fa_append on `stream`: the new token takes row `slot` of k_full / v_full; with
    `evict` the row's old token is first folded into ck / cv / k_keep / v_keep as middle token
    number n_mid.  Everything is updated in place."""
    B, Hkv, D = k_new.shape
    W = k_full.shape[2]
    Dkc = ck.shape[-1] if ck is not None else 0
    Dvc = cv.shape[-1] if cv is not None else 0
    st = lib.fa_append(_ptr(k_new), _ptr(v_new), _dtype_code(k_new), B, Hkv, D,
                       _ptr(k_full), _ptr(v_full), W, full_stride_bh, int(slot), 1 if evict else 0,
                       _ptr(kmask), Dkc, _ptr(vmask), Dvc, M, T, n_mid,
                       _ptr(ck), _ptr(cv), _ptr(k_keep), kk_stride_bh, _ptr(v_keep), vk_stride_bh,
                       _stream_ptr(stream))
    if st != FA_OK:
        raise FourierAttnError(st, "fa_append")


def fa_append_varlen(k_new, v_new, k_full, v_full, seq_slot, kmask, vmask, M, T, seq_nmid, n_cap,
                     ck, cv, k_keep, v_keep, stream=None, kk_stride_bh=0, vk_stride_bh=0, full_stride_bh=0):
    """Enqueue fa_append_varlen: `seq_slot` / `seq_nmid` are int32 device tensors [B] with each sequence's
    ring row and fold position (negative fold position: the row is written, nothing is folded)."""
    B, Hkv, D = k_new.shape
    W = k_full.shape[2]
    Dkc = ck.shape[-1] if ck is not None else 0
    Dvc = cv.shape[-1] if cv is not None else 0
    for t in (seq_slot, seq_nmid):
        if t.dtype != torch.int32 or t.numel() != B or not t.is_contiguous():
            raise ValueError("seq_slot / seq_nmid must be contiguous int32 tensors of B entries")
    st = lib.fa_append_varlen(_ptr(k_new), _ptr(v_new), _dtype_code(k_new), B, Hkv, D,
                              _ptr(k_full), _ptr(v_full), W, full_stride_bh, _ptr(seq_slot),
                              _ptr(kmask), Dkc, _ptr(vmask), Dvc, M, T, _ptr(seq_nmid), int(n_cap),
                              _ptr(ck), _ptr(cv), _ptr(k_keep), kk_stride_bh, _ptr(v_keep), vk_stride_bh,
                              _stream_ptr(stream))
    if st != FA_OK:
        raise FourierAttnError(st, "fa_append_varlen")


def select_workspace_bytes(dtype_code, B, H, N, D, M) -> int:
    return int(lib.fa_select_workspace_bytes(dtype_code, B, H, N, D, M))


def fa_select_dims(x, M, Dc, want_mse=True, workspace=None, stream=None):
    """Enqueue fa_select_dims on `stream` for x [B,H,N,D]; returns (dim_mask uint8 [B,H,D],
    mse fp32 [B,H,D] or None)."""
    B, H, N, D = x.shape
    dev = x.device
    mask = torch.empty((B, H, D), dtype=torch.uint8, device=dev)
    mse = torch.empty((B, H, D), dtype=torch.float32, device=dev) if want_mse else None
    if workspace is None:
        need = select_workspace_bytes(_dtype_code(x), B, H, N, D, M)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    st = lib.fa_select_dims(_ptr(x), _dtype_code(x), x.stride(0), x.stride(1), x.stride(2), B, H, N, D, M, Dc,
                            _ptr(mask), _ptr(mse), _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if st != FA_OK:
        raise FourierAttnError(st, "fa_select_dims")
    return mask, mse


def legt_workspace_bytes(B, H, N, D, M) -> int:
    return int(lib.fa_legt_workspace_bytes(B, H, N, D, M))


def fa_legt(x, M, workspace=None, stream=None, want_mse=True):
    """Enqueue fa_legt_compress (and fa_legt_mse) on `stream` for x [B,H,N,D]: returns (coeffs fp32
    [B,H,M,D], mse fp32 [B,H,D] or None)."""
    B, H, N, D = x.shape
    dev = x.device
    coeffs = torch.empty((B, H, M, D), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(legt_workspace_bytes(B, H, N, D, M), 256), dtype=torch.uint8, device=dev)
    st = lib.fa_legt_compress(_ptr(x), _dtype_code(x), x.stride(0), x.stride(1), x.stride(2), B, H, N, D, M,
                              _ptr(coeffs), _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if st != FA_OK:
        raise FourierAttnError(st, "fa_legt_compress")
    mse = None
    if want_mse:
        mse = torch.empty((B, H, D), dtype=torch.float32, device=dev)
        st = lib.fa_legt_mse(_ptr(x), _dtype_code(x), x.stride(0), x.stride(1), x.stride(2), B, H, N, D, M,
                             _ptr(coeffs), _ptr(mse), _ptr(workspace), workspace.numel(), _stream_ptr(stream))
        if st != FA_OK:
            raise FourierAttnError(st, "fa_legt_mse")
    return coeffs, mse


def fa_decode_mq(q, ck, kmask, cv, vmask, M, T, t0, N, k_keep, v_keep, k_full, v_full,
                 scale=0.0, num_splits=0, out=None, workspace=None, stream=None):
    """Enqueue fa_decode_mq on `stream`: q [B, Hkv, Tq, G, D] -> out fp32 of the same shape; the last
    Tq rows of k_full / v_full are the new tokens."""
    B, Hkv, Tq, G, D = q.shape
    Hq = Hkv * G
    Dkc = ck.shape[-1] if ck is not None else 0
    Dvc = cv.shape[-1] if cv is not None else 0
    W = k_full.shape[2]
    dev = q.device
    if out is None:
        out = torch.empty((B, Hkv, Tq, G, D), dtype=torch.float32, device=dev)
    if workspace is None:
        need = decode_workspace_bytes(B, Hq * Tq, Hkv, D, Dkc, Dvc, M, N, W, num_splits)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    st = lib.fa_decode_mq(_ptr(q), _dtype_code(q), B, Tq, Hq, Hkv, D, _ptr(ck), _ptr(kmask), Dkc, _ptr(cv),
                          _ptr(vmask), Dvc, M, T, t0, N, _ptr(k_keep), 0, _ptr(v_keep), 0, _ptr(k_full),
                          _ptr(v_full), W, 0, float(scale), num_splits, _ptr(out), _ptr(workspace),
                          workspace.numel(), _stream_ptr(stream))
    if st != FA_OK:
        raise FourierAttnError(st, "fa_decode_mq")
    return out


def compress_kv_workspace_bytes(B, H, N, D, Dkc, Dvc, M, dtype=None) -> int:
    if dtype is None:
        return int(lib.fa_compress_kv_workspace_bytes(B, H, N, D, Dkc, Dvc, M))
    code = dtype if isinstance(dtype, int) else (FA_F32 if dtype == torch.float32 else FA_BF16)
    return int(lib.fa_compress_kv_workspace_bytes_for(code, B, H, N, D, Dkc, Dvc, M))


def fa_compress_kv(k, v, kmask, vmask, Dkc, Dvc, M, T, t0=0, accumulate=False, ck=None, cv=None,
                   k_keep=None, v_keep=None, keep_offset=0, workspace=None, stream=None, kernel_ms=None):
    """Enqueue fa_compress_kv on `stream`: K and V segments [B,H,N,D] of the same tokens.  Returns
    (ck, k_keep rows layout, cv, v_keep groups-of-8-tokens layout).  With `kernel_ms` (a list) the timed,
    synchronous entry point is used and (projection, reduction) milliseconds appended."""
    B, H, N, D = k.shape
    assert v.shape == k.shape and v.stride() == k.stride() and v.dtype == k.dtype
    dev = k.device
    n_tok = keep_offset + N
    if ck is None:
        ck = torch.empty((B, H, M, Dkc), dtype=torch.float32, device=dev)
    if cv is None:
        cv = torch.empty((B, H, M, Dvc), dtype=torch.float32, device=dev)
    if k_keep is None:
        k_keep = torch.empty((B, H, n_tok, keep_rows_pitch(D - Dkc)), dtype=k.dtype, device=dev)
    if v_keep is None:
        v_keep = torch.zeros((B, H, tok8_numel(n_tok, D - Dvc)), dtype=k.dtype, device=dev)
    if workspace is None:
        workspace = torch.empty(max(compress_kv_workspace_bytes(B, H, N, D, Dkc, Dvc, M, k.dtype), 256), dtype=torch.uint8,
                                device=dev)
    args = (_ptr(k), _ptr(v), _dtype_code(k), k.stride(0), k.stride(1), k.stride(2), B, H, N, D,
            _ptr(kmask), Dkc, _ptr(vmask), Dvc, M, T, t0, int(bool(accumulate)), _ptr(ck), _ptr(cv),
            _ptr(k_keep), 0, _ptr(v_keep), 0, keep_offset, _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if kernel_ms is None:
        st = lib.fa_compress_kv(*args)
    else:
        ms = (ctypes.c_float * 2)()
        st = lib.fa_compress_kv_timed(*args, ms)
        kernel_ms.extend(ms)
    if st != FA_OK:
        raise FourierAttnError(st, "fa_compress_kv")
    return ck, k_keep, cv, v_keep

