"""MI355X-native SALR linear layer: thin Python binding over the C boundary in ``include/salr.h``.

The three operations keep their C names (``salr_encode_bitmap``, ``salr_decode``,
``salr_sparse_lowrank_linear``); this module only marshals arguments: torch CUDA tensors supply
device memory and the current stream, every step of the computation runs in the HIP kernels of
``libsalr_hip.so``.  There is no CPU or PyTorch fallback: a missing library is an ImportError.

bf16 tensors may be given as ``torch.bfloat16`` or as their raw patterns (``torch.int16`` /
``torch.uint16``); bitmap and row offsets are ``torch.int32`` / ``torch.uint32``.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsalr_hip.so")

SALR_OK, SALR_ERR_INVALID_ARG, SALR_ERR_SHAPE, SALR_ERR_CAPACITY, SALR_ERR_UNSUPPORTED, SALR_ERR_HIP = range(6)

_lib = None
_vp = ctypes.c_void_p
_i64 = ctypes.c_int64


class SalrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        msg = lib().salr_status_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Built by ``paper_2601_16991_amd/build.py`` (or __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python paper_2601_16991_amd/build.py` first")
        L = ctypes.CDLL(LIB_PATH)
        L.salr_status_string.restype = ctypes.c_char_p
        L.salr_status_string.argtypes = [ctypes.c_int]
        L.salr_bitmap_words_per_row.restype = _i64
        L.salr_bitmap_words_per_row.argtypes = [_i64]
        L.salr_magnitude_mask_rows.restype = ctypes.c_int
        L.salr_magnitude_mask_rows.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp]
        L.salr_magnitude_mask_nm.restype = ctypes.c_int
        L.salr_magnitude_mask_nm.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, _vp]
        L.salr_encode_bitmap.restype = ctypes.c_int
        L.salr_encode_bitmap.argtypes = [_vp, _i64, _i64, _vp, _vp, _i64, _vp, _vp]
        L.salr_decode.restype = ctypes.c_int
        L.salr_decode.argtypes = [_vp, _vp, _vp, _i64, _i64, _vp, _vp]
        L.salr_linear_workspace_bytes.restype = ctypes.c_size_t
        L.salr_linear_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64]
        L.salr_linear_workspace_bytes_min.restype = ctypes.c_size_t
        L.salr_linear_workspace_bytes_min.argtypes = [_i64, _i64, _i64, _i64]
        L.salr_sparse_lowrank_linear.restype = ctypes.c_int
        L.salr_sparse_lowrank_linear.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _vp,
                                                 ctypes.c_size_t, _vp]
        L.salr_slice_table_bytes.restype = ctypes.c_size_t
        L.salr_slice_table_bytes.argtypes = [_i64, _i64]
        L.salr_build_slice_table.restype = ctypes.c_int
        L.salr_build_slice_table.argtypes = [_vp, _vp, _i64, _i64, _vp, ctypes.c_size_t, _vp]
        L.salr_sparse_lowrank_linear_prepared.restype = ctypes.c_int
        L.salr_sparse_lowrank_linear_prepared.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _vp,
                                                          ctypes.c_size_t, _vp]
        L.salr_sparse_lowrank_linear_noalloc.restype = ctypes.c_int
        L.salr_sparse_lowrank_linear_noalloc.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _vp]
        L.salr_nf4_quantize_values.restype = ctypes.c_int
        L.salr_nf4_quantize_values.argtypes = [_vp, _i64, _vp, _vp, _vp]
        L.salr_nf4_dequantize_values.restype = ctypes.c_int
        L.salr_nf4_dequantize_values.argtypes = [_vp, _vp, _i64, _vp, _vp]
        L.salr_qsalr_linear_workspace_bytes.restype = ctypes.c_size_t
        L.salr_qsalr_linear_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, _i64]
        L.salr_qsalr_linear.restype = ctypes.c_int
        L.salr_qsalr_linear.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _i64, _vp, _vp, _i64, _vp, _vp,
                                        ctypes.c_size_t, _vp]
        L.salr_bitmap_is_2of4.restype = ctypes.c_int
        L.salr_bitmap_is_2of4.argtypes = [_vp, _i64, _i64, _vp, _vp]
        L.salr_linear_2of4_workspace_bytes.restype = ctypes.c_size_t
        L.salr_linear_2of4_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64]
        L.salr_sparse_lowrank_linear_2of4.restype = ctypes.c_int
        L.salr_sparse_lowrank_linear_2of4.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _vp,
                                                      ctypes.c_size_t, _vp]
        L.salr_residual.restype = ctypes.c_int
        L.salr_residual.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp]
        L.salr_concat_adapters.restype = ctypes.c_int
        L.salr_concat_adapters.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_i64), _i64, _i64, _i64,
                                           _vp, _vp, _vp]
        L.salr_residual_adapter_workspace_bytes.restype = ctypes.c_size_t
        L.salr_residual_adapter_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64]
        L.salr_residual_adapter.restype = ctypes.c_int
        L.salr_residual_adapter.argtypes = [_vp, _i64, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        L.salr_linear_backward_workspace_bytes.restype = ctypes.c_size_t
        L.salr_linear_backward_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, ctypes.c_int, ctypes.c_int]
        L.salr_sparse_lowrank_linear_backward.restype = ctypes.c_int
        L.salr_sparse_lowrank_linear_backward.argtypes = [_vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _i64, _vp, _vp,
                                                          _vp, _vp, ctypes.c_size_t, _vp]
        L.salr_set_kernel_timing_events.restype = None
        L.salr_set_kernel_timing_events.argtypes = [_vp, _vp]
        _lib = L
    return _lib


_BF16_TYPES = (torch.bfloat16, torch.int16, torch.uint16)
_U32_TYPES = (torch.int32, torch.uint32)


def _ptr(t: Optional[torch.Tensor], kinds, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if t.dtype not in kinds:
        raise TypeError(f"{name}: dtype {t.dtype} not in {kinds}")
    if not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous")
    return t.data_ptr() if t.numel() > 0 else None


def _stream(stream) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check(status: int, where: str) -> None:
    if status != SALR_OK:
        raise SalrError(status, where)


def salr_bitmap_words_per_row(cols: int) -> int:
    return int(lib().salr_bitmap_words_per_row(cols))


def salr_magnitude_mask_rows(w: torch.Tensor, keep: int, w_hat: torch.Tensor, stream=None) -> None:
    """Enqueue the per-row magnitude mask: w_hat = w with all but the `keep` largest |w| of each row zeroed."""
    rows, cols = w.shape
    if tuple(w_hat.shape) != (rows, cols):
        raise ValueError("w_hat shape")
    st = lib().salr_magnitude_mask_rows(_ptr(w, _BF16_TYPES, "w"), rows, cols, keep,
                                        _ptr(w_hat, _BF16_TYPES, "w_hat"), _stream(stream))
    _check(st, "salr_magnitude_mask_rows")


def salr_magnitude_mask_nm(w: torch.Tensor, n_keep: int, m_group: int, w_hat: torch.Tensor, stream=None) -> None:
    """Enqueue the N:M mask: the n_keep largest |w| of every m_group consecutive columns survive."""
    rows, cols = w.shape
    if tuple(w_hat.shape) != (rows, cols):
        raise ValueError("w_hat shape")
    st = lib().salr_magnitude_mask_nm(_ptr(w, _BF16_TYPES, "w"), rows, cols, n_keep, m_group,
                                      _ptr(w_hat, _BF16_TYPES, "w_hat"), _stream(stream))
    _check(st, "salr_magnitude_mask_nm")


def salr_encode_bitmap(w_dense: torch.Tensor, bitmap: torch.Tensor, values: Optional[torch.Tensor],
                       row_offsets: torch.Tensor, stream=None) -> None:
    """Enqueue the encoder.  ``values`` None = count only; its length is the capacity."""
    rows, cols = w_dense.shape
    cap = 0 if values is None else values.numel()
    st = lib().salr_encode_bitmap(_ptr(w_dense, _BF16_TYPES, "w_dense"), rows, cols, _ptr(bitmap, _U32_TYPES, "bitmap"),
                                  _ptr(values, _BF16_TYPES, "values"), cap, _ptr(row_offsets, _U32_TYPES, "row_offsets"),
                                  _stream(stream))
    _check(st, "salr_encode_bitmap")


def salr_decode(bitmap: torch.Tensor, values: torch.Tensor, row_offsets: torch.Tensor, rows: int, cols: int,
                w_dense_out: torch.Tensor, stream=None) -> None:
    st = lib().salr_decode(_ptr(bitmap, _U32_TYPES, "bitmap"), _ptr(values, _BF16_TYPES, "values"),
                           _ptr(row_offsets, _U32_TYPES, "row_offsets"), rows, cols,
                           _ptr(w_dense_out, _BF16_TYPES, "w_dense_out"), _stream(stream))
    _check(st, "salr_decode")


def salr_linear_workspace_bytes(M: int, K: int, N: int, R: int) -> int:
    return int(lib().salr_linear_workspace_bytes(M, K, N, R))


def salr_linear_workspace_bytes_min(M: int, K: int, N: int, R: int) -> int:
    return int(lib().salr_linear_workspace_bytes_min(M, K, N, R))


def salr_sparse_lowrank_linear(x: torch.Tensor, bitmap: torch.Tensor, values: torch.Tensor,
                               row_offsets: torch.Tensor, a_cat: Optional[torch.Tensor],
                               b_cat: Optional[torch.Tensor], y: torch.Tensor,
                               workspace: Optional[torch.Tensor], stream=None) -> None:
    """Enqueue Y = X What^T + (X A_cat) B_cat.  Shapes: x [M,K], bitmap [N,K/32], a_cat [K,R], b_cat [R,N], y [M,N]."""
    M, K = x.shape
    N = y.shape[1]
    R = 0 if a_cat is None else a_cat.shape[1]
    if y.shape[0] != M or bitmap.shape[0] != N or row_offsets.numel() != N + 1:
        raise ValueError("inconsistent shapes")
    if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
        raise ValueError("adapter shapes")
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().salr_sparse_lowrank_linear(_ptr(x, _BF16_TYPES, "x"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"),
                                          _ptr(values, _BF16_TYPES, "values"),
                                          _ptr(row_offsets, _U32_TYPES, "row_offsets"),
                                          _ptr(a_cat, _BF16_TYPES, "a_cat"), _ptr(b_cat, _BF16_TYPES, "b_cat"), R,
                                          _ptr(y, _BF16_TYPES, "y"), ws_ptr, ws_bytes, _stream(stream))
    _check(st, "salr_sparse_lowrank_linear")


def salr_slice_table_bytes(N: int, K: int) -> int:
    return int(lib().salr_slice_table_bytes(N, K))


def salr_build_slice_table(bitmap: torch.Tensor, row_offsets: torch.Tensor, K: int, slice_table: torch.Tensor,
                           stream=None) -> None:
    """Enqueue the layer's slice table: slice_table int32/uint32 [N, 8, 2] (see include/salr.h)."""
    N = bitmap.shape[0]
    _check(lib().salr_build_slice_table(_ptr(bitmap, _U32_TYPES, "bitmap"), _ptr(row_offsets, _U32_TYPES, "row_offsets"),
                                        N, K, _ptr(slice_table, _U32_TYPES, "slice_table"),
                                        slice_table.numel() * slice_table.element_size(), _stream(stream)),
           "salr_build_slice_table")


def salr_sparse_lowrank_linear_prepared(x: torch.Tensor, bitmap: torch.Tensor, values: torch.Tensor,
                                        row_offsets: torch.Tensor, slice_table: torch.Tensor,
                                        a_cat: Optional[torch.Tensor], b_cat: Optional[torch.Tensor], y: torch.Tensor,
                                        workspace: Optional[torch.Tensor], stream=None) -> None:
    """salr_sparse_lowrank_linear with the layer's slice table as one more input."""
    M, K = x.shape
    N = y.shape[1]
    R = 0 if a_cat is None else a_cat.shape[1]
    if y.shape[0] != M or bitmap.shape[0] != N or row_offsets.numel() != N + 1 or slice_table.numel() != N * 16:
        raise ValueError("inconsistent shapes")
    if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
        raise ValueError("adapter shapes")
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().salr_sparse_lowrank_linear_prepared(
        _ptr(x, _BF16_TYPES, "x"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"), _ptr(values, _BF16_TYPES, "values"),
        _ptr(row_offsets, _U32_TYPES, "row_offsets"), _ptr(slice_table, _U32_TYPES, "slice_table"),
        _ptr(a_cat, _BF16_TYPES, "a_cat"), _ptr(b_cat, _BF16_TYPES, "b_cat"), R, _ptr(y, _BF16_TYPES, "y"), ws_ptr, ws_bytes,
        _stream(stream))
    _check(st, "salr_sparse_lowrank_linear_prepared")


def salr_nf4_quantize_values(values: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor, stream=None) -> None:
    """Enqueue QSALR's coding of the packed values: codes uint8 [ceil(n/2)], scales bf16 [ceil(n/64)]."""
    n = values.numel()
    if codes.dtype != torch.uint8 or codes.numel() < (n + 1) // 2 or scales.numel() < (n + 63) // 64:
        raise ValueError("codes must be uint8 [ceil(n/2)] and scales [ceil(n/64)]")
    _check(lib().salr_nf4_quantize_values(_ptr(values, _BF16_TYPES, "values"), n, _ptr(codes, (torch.uint8,), "codes"),
                                          _ptr(scales, _BF16_TYPES, "scales"), _stream(stream)), "salr_nf4_quantize_values")


def salr_nf4_dequantize_values(codes: torch.Tensor, scales: torch.Tensor, count: int, values_out: torch.Tensor,
                               stream=None) -> None:
    """Enqueue the inverse: values_out [count] bf16 (its storage padded to a multiple of 8 elements)."""
    if codes.numel() < (count + 1) // 2 or scales.numel() < (count + 63) // 64 or values_out.numel() < count:
        raise ValueError("buffers too short for count")
    _check(lib().salr_nf4_dequantize_values(_ptr(codes, (torch.uint8,), "codes"), _ptr(scales, _BF16_TYPES, "scales"), count,
                                            _ptr(values_out, _BF16_TYPES, "values_out"), _stream(stream)),
           "salr_nf4_dequantize_values")


def salr_qsalr_linear_workspace_bytes(M: int, K: int, N: int, R: int, nnz: int) -> int:
    return int(lib().salr_qsalr_linear_workspace_bytes(M, K, N, R, nnz))


def salr_qsalr_linear(x: torch.Tensor, bitmap: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor,
                      row_offsets: torch.Tensor, nnz: int, a_cat: Optional[torch.Tensor], b_cat: Optional[torch.Tensor],
                      y: torch.Tensor, workspace: Optional[torch.Tensor], stream=None) -> None:
    """Enqueue Y = X decode(bitmap, dequantised codes)^T + (X A_cat) B_cat."""
    M, K = x.shape
    N = y.shape[1]
    R = 0 if a_cat is None else a_cat.shape[1]
    if y.shape[0] != M or bitmap.shape[0] != N or row_offsets.numel() != N + 1:
        raise ValueError("inconsistent shapes")
    if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
        raise ValueError("adapter shapes")
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().salr_qsalr_linear(_ptr(x, _BF16_TYPES, "x"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"),
                                 _ptr(codes, (torch.uint8,), "codes"), _ptr(scales, _BF16_TYPES, "scales"),
                                 _ptr(row_offsets, _U32_TYPES, "row_offsets"), nnz, _ptr(a_cat, _BF16_TYPES, "a_cat"),
                                 _ptr(b_cat, _BF16_TYPES, "b_cat"), R, _ptr(y, _BF16_TYPES, "y"), ws_ptr, ws_bytes,
                                 _stream(stream))
    _check(st, "salr_qsalr_linear")


def codes_alloc(count: int, device) -> torch.Tensor:
    """A buffer for the 4-bit codes of `count` values whose storage is whole 16-byte vectors (salr_qsalr_linear reads
    the codes with vector loads)."""
    nbytes = (count + 1) // 2
    return torch.empty(max((nbytes + 15) // 16 * 16, 16), dtype=torch.uint8, device=device)[:nbytes]


def nf4_quantize(values: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    n = values.numel()
    codes = codes_alloc(n, values.device)
    scales = torch.empty(max((n + 63) // 64, 1), dtype=torch.int16, device=values.device)[:(n + 63) // 64]
    salr_nf4_quantize_values(values, codes, scales)
    return codes, scales


def nf4_dequantize(codes: torch.Tensor, scales: torch.Tensor, count: int) -> torch.Tensor:
    out = values_alloc(count, codes.device)
    salr_nf4_dequantize_values(codes, scales, count, out)
    return out


def qsalr_linear(x, bitmap, codes, scales, row_offsets, nnz, a_cat, b_cat) -> torch.Tensor:
    M, K = x.shape
    N = bitmap.shape[0]
    R = 0 if a_cat is None else a_cat.shape[1]
    y = torch.empty((M, N), dtype=x.dtype, device=x.device)
    ws = torch.empty(max(salr_qsalr_linear_workspace_bytes(M, K, N, R, nnz), 256), dtype=torch.uint8, device=x.device)
    salr_qsalr_linear(x, bitmap, codes, scales, row_offsets, nnz, a_cat, b_cat, y, ws)
    return y


NOALLOC_SCRATCH_BYTES = 16 * 1024 * 1024   # SALR_NOALLOC_SCRATCH_BYTES of include/salr.h


def salr_sparse_lowrank_linear_noalloc(x: torch.Tensor, bitmap: torch.Tensor, values: torch.Tensor,
                                       row_offsets: torch.Tensor, a_cat: Optional[torch.Tensor],
                                       b_cat: Optional[torch.Tensor], y: torch.Tensor, stream=None) -> None:
    """Enqueue Y = X What^T + (X A_cat) B_cat with the library's own fixed scratch array in place of a workspace."""
    M, K = x.shape
    N = y.shape[1]
    R = 0 if a_cat is None else a_cat.shape[1]
    if y.shape[0] != M or bitmap.shape[0] != N or row_offsets.numel() != N + 1:
        raise ValueError("inconsistent shapes")
    if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
        raise ValueError("adapter shapes")
    st = lib().salr_sparse_lowrank_linear_noalloc(_ptr(x, _BF16_TYPES, "x"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"),
                                                  _ptr(values, _BF16_TYPES, "values"),
                                                  _ptr(row_offsets, _U32_TYPES, "row_offsets"),
                                                  _ptr(a_cat, _BF16_TYPES, "a_cat"), _ptr(b_cat, _BF16_TYPES, "b_cat"), R,
                                                  _ptr(y, _BF16_TYPES, "y"), _stream(stream))
    _check(st, "salr_sparse_lowrank_linear_noalloc")


def salr_bitmap_is_2of4(bitmap: torch.Tensor, result: torch.Tensor, stream=None) -> None:
    """Enqueue the check: result[0] (one uint32 on the device) = 1 iff every aligned group of four columns has two set bits."""
    rows, wpr = bitmap.shape
    st = lib().salr_bitmap_is_2of4(_ptr(bitmap, _U32_TYPES, "bitmap"), rows, wpr * 32, _ptr(result, _U32_TYPES, "result"),
                                   _stream(stream))
    _check(st, "salr_bitmap_is_2of4")


def salr_linear_2of4_workspace_bytes(M: int, K: int, N: int, R: int) -> int:
    return int(lib().salr_linear_2of4_workspace_bytes(M, K, N, R))


def salr_sparse_lowrank_linear_2of4(x: torch.Tensor, bitmap: torch.Tensor, values: torch.Tensor,
                                    row_offsets: torch.Tensor, a_cat: Optional[torch.Tensor],
                                    b_cat: Optional[torch.Tensor], y: torch.Tensor,
                                    workspace: Optional[torch.Tensor], stream=None) -> None:
    """Enqueue Y = X What^T + (X A_cat) B_cat for a weight that passes salr_bitmap_is_2of4 (not checked here)."""
    M, K = x.shape
    N = y.shape[1]
    R = 0 if a_cat is None else a_cat.shape[1]
    if y.shape[0] != M or bitmap.shape[0] != N or row_offsets.numel() != N + 1:
        raise ValueError("inconsistent shapes")
    if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
        raise ValueError("adapter shapes")
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().salr_sparse_lowrank_linear_2of4(_ptr(x, _BF16_TYPES, "x"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"),
                                               _ptr(values, _BF16_TYPES, "values"),
                                               _ptr(row_offsets, _U32_TYPES, "row_offsets"),
                                               _ptr(a_cat, _BF16_TYPES, "a_cat"), _ptr(b_cat, _BF16_TYPES, "b_cat"), R,
                                               _ptr(y, _BF16_TYPES, "y"), ws_ptr, ws_bytes, _stream(stream))
    _check(st, "salr_sparse_lowrank_linear_2of4")


def salr_linear_backward_workspace_bytes(M: int, K: int, N: int, R: int, want_dx: bool, want_dadb: bool) -> int:
    return int(lib().salr_linear_backward_workspace_bytes(M, K, N, R, int(want_dx), int(want_dadb)))


def salr_sparse_lowrank_linear_backward(x: Optional[torch.Tensor], dy: torch.Tensor, bitmap: torch.Tensor,
                                        values: torch.Tensor, row_offsets: torch.Tensor, a_cat: Optional[torch.Tensor],
                                        b_cat: Optional[torch.Tensor], dx: Optional[torch.Tensor],
                                        da: Optional[torch.Tensor], db: Optional[torch.Tensor],
                                        workspace: Optional[torch.Tensor], stream=None) -> None:
    """Enqueue dX = dY What + (dY B_cat^T) A_cat^T, dA = X^T (dY B_cat^T), dB = (X A_cat)^T dY; None = not computed."""
    M, N = dy.shape
    K = bitmap.shape[1] * 32
    R = 0 if a_cat is None else a_cat.shape[1]
    if bitmap.shape[0] != N or row_offsets.numel() != N + 1:
        raise ValueError("inconsistent shapes")
    if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
        raise ValueError("adapter shapes")
    for name, t, shape in (("x", x, (M, K)), ("dx", dx, (M, K)), ("da", da, (K, R)), ("db", db, (R, N))):
        if t is not None and tuple(t.shape) != shape:
            raise ValueError(f"{name} must be {shape}")
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = lib().salr_sparse_lowrank_linear_backward(
        _ptr(x, _BF16_TYPES, "x"), _ptr(dy, _BF16_TYPES, "dy"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"),
        _ptr(values, _BF16_TYPES, "values"), _ptr(row_offsets, _U32_TYPES, "row_offsets"),
        _ptr(a_cat, _BF16_TYPES, "a_cat"), _ptr(b_cat, _BF16_TYPES, "b_cat"), R, _ptr(dx, _BF16_TYPES, "dx"),
        _ptr(da, _BF16_TYPES, "da"), _ptr(db, _BF16_TYPES, "db"), ws_ptr, ws_bytes, _stream(stream))
    _check(st, "salr_sparse_lowrank_linear_backward")


def linear_backward(x, dy, bitmap, values, row_offsets, a_cat, b_cat, need_dx=True, need_dadb=True):
    """(dx, da, db); entries not asked for (or without adapters) are None."""
    M, N = dy.shape
    K = bitmap.shape[1] * 32
    R = 0 if a_cat is None else a_cat.shape[1]
    dev = dy.device
    dx = torch.empty((M, K), dtype=dy.dtype, device=dev) if need_dx else None
    da = torch.empty((K, R), dtype=dy.dtype, device=dev) if need_dadb and R else None
    db = torch.empty((R, N), dtype=dy.dtype, device=dev) if need_dadb and R else None
    need = salr_linear_backward_workspace_bytes(M, K, N, R, need_dx, need_dadb and R > 0)
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    salr_sparse_lowrank_linear_backward(x, dy, bitmap, values, row_offsets, a_cat, b_cat, dx, da, db, ws)
    return dx, da, db


class PreparedLinear:
    """The argument list of one salr_sparse_lowrank_linear call, marshalled once: ``run()`` is then a
    single foreign call on the stream that is current at that moment (for launch-bound loops)."""

    def __init__(self, x, bitmap, values, row_offsets, a_cat, b_cat, y, workspace, two_of_four=False, slice_table=None):
        M, K = x.shape
        N = y.shape[1]
        R = 0 if a_cat is None else a_cat.shape[1]
        if y.shape[0] != M or bitmap.shape[0] != N or row_offsets.numel() != N + 1:
            raise ValueError("inconsistent shapes")
        if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
            raise ValueError("adapter shapes")
        if slice_table is not None and (two_of_four or slice_table.numel() != N * 16):
            raise ValueError("slice table")
        self._keep = (x, bitmap, values, row_offsets, a_cat, b_cat, y, workspace, slice_table)
        ws_ptr = None if workspace is None else workspace.data_ptr()
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        table = () if slice_table is None else (_ptr(slice_table, _U32_TYPES, "slice_table"),)
        self._args = (_ptr(x, _BF16_TYPES, "x"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"),
                      _ptr(values, _BF16_TYPES, "values"), _ptr(row_offsets, _U32_TYPES, "row_offsets")) + table + (
                      _ptr(a_cat, _BF16_TYPES, "a_cat"), _ptr(b_cat, _BF16_TYPES, "b_cat"), R,
                      _ptr(y, _BF16_TYPES, "y"), ws_ptr, ws_bytes)
        self._fn = (lib().salr_sparse_lowrank_linear_prepared if slice_table is not None else
                    lib().salr_sparse_lowrank_linear_2of4 if two_of_four else lib().salr_sparse_lowrank_linear)

    def run(self, stream_handle: Optional[int] = None) -> None:
        st = self._fn(*self._args, stream_handle)
        if st != SALR_OK:
            raise SalrError(st, "salr_sparse_lowrank_linear")


class PreparedQsalrLinear:
    """The argument list of one salr_qsalr_linear call, marshalled once (see PreparedLinear)."""

    def __init__(self, x, bitmap, codes, scales, row_offsets, nnz, a_cat, b_cat, y, workspace):
        M, K = x.shape
        N = y.shape[1]
        R = 0 if a_cat is None else a_cat.shape[1]
        if y.shape[0] != M or bitmap.shape[0] != N or row_offsets.numel() != N + 1:
            raise ValueError("inconsistent shapes")
        if R and (tuple(a_cat.shape) != (K, R) or tuple(b_cat.shape) != (R, N)):
            raise ValueError("adapter shapes")
        if codes.numel() != (nnz + 1) // 2 or scales.numel() != (nnz + 63) // 64:
            raise ValueError("codes / scales do not match nnz")
        self._keep = (x, bitmap, codes, scales, row_offsets, a_cat, b_cat, y, workspace)
        ws_ptr = None if workspace is None else workspace.data_ptr()
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        self._args = (_ptr(x, _BF16_TYPES, "x"), M, K, N, _ptr(bitmap, _U32_TYPES, "bitmap"),
                      _ptr(codes, (torch.uint8,), "codes"), _ptr(scales, _BF16_TYPES, "scales"),
                      _ptr(row_offsets, _U32_TYPES, "row_offsets"), nnz, _ptr(a_cat, _BF16_TYPES, "a_cat"),
                      _ptr(b_cat, _BF16_TYPES, "b_cat"), R, _ptr(y, _BF16_TYPES, "y"), ws_ptr, ws_bytes)

    def run(self, stream_handle: Optional[int] = None) -> None:
        st = lib().salr_qsalr_linear(*self._args, stream_handle)
        if st != SALR_OK:
            raise SalrError(st, "salr_qsalr_linear")


def salr_set_kernel_timing_events(start_event: Optional[int], stop_event: Optional[int]) -> None:
    """Measurement hook: hipEvent_t handles (as integers) recorded around the fused kernel; None, None = off."""
    lib().salr_set_kernel_timing_events(start_event, stop_event)


# ---------------------------------------------------------------------------------------------------
# Convenience wrappers: allocate the outputs with torch, then call the entry points above.
# ---------------------------------------------------------------------------------------------------

def values_alloc(nnz: int, device) -> torch.Tensor:
    """A packed-values buffer of nnz elements whose storage is padded to a multiple of 16 bytes."""
    padded = (nnz + 7) // 8 * 8
    return torch.empty(max(padded, 8), dtype=torch.int16, device=device)[:nnz]


def mask_rows(w: torch.Tensor, keep: int) -> torch.Tensor:
    w_hat = torch.empty_like(w)
    salr_magnitude_mask_rows(w, keep, w_hat)
    return w_hat


def mask_nm(w: torch.Tensor, n_keep: int, m_group: int) -> torch.Tensor:
    w_hat = torch.empty_like(w)
    salr_magnitude_mask_nm(w, n_keep, m_group, w_hat)
    return w_hat


def salr_residual(w: torch.Tensor, w_hat: torch.Tensor, e: torch.Tensor, stream=None) -> None:
    """Enqueue E = W - What (bf16, [rows, cols])."""
    if w.shape != w_hat.shape or w.shape != e.shape or w.dim() != 2:
        raise ValueError("w, w_hat and e must be matrices of one shape")
    rows, cols = w.shape
    _check(lib().salr_residual(_ptr(w, _BF16_TYPES, "w"), _ptr(w_hat, _BF16_TYPES, "w_hat"), rows, cols,
                               _ptr(e, _BF16_TYPES, "e"), _stream(stream)), "salr_residual")


def salr_concat_adapters(a_list: Sequence[torch.Tensor], b_list: Sequence[torch.Tensor], a_cat: torch.Tensor,
                         b_cat: torch.Tensor, stream=None) -> None:
    """Enqueue A_cat = [A_1 ... A_n] ([K, R]) and B_cat = [B_1; ...; B_n] ([R, N])."""
    n = len(a_list)
    if len(b_list) != n:
        raise ValueError("as many A_i as B_i")
    K, N = a_cat.shape[0], b_cat.shape[1]
    ranks = []
    for i, (a, b) in enumerate(zip(a_list, b_list)):
        if a.dim() != 2 or b.dim() != 2 or a.shape[0] != K or b.shape[1] != N or a.shape[1] != b.shape[0]:
            raise ValueError(f"adapter {i}: shapes {tuple(a.shape)} {tuple(b.shape)}")
        ranks.append(a.shape[1])
    if a_cat.shape[1] != sum(ranks) or b_cat.shape[0] != sum(ranks):
        raise ValueError("a_cat / b_cat do not have sum(ranks) columns / rows")
    pa = (_vp * max(n, 1))(*[_ptr(a, _BF16_TYPES, "A_i") for a in a_list])
    pb = (_vp * max(n, 1))(*[_ptr(b, _BF16_TYPES, "B_i") for b in b_list])
    rk = (_i64 * max(n, 1))(*ranks)
    _check(lib().salr_concat_adapters(pa, pb, rk, n, K, N, _ptr(a_cat, _BF16_TYPES, "a_cat"),
                                      _ptr(b_cat, _BF16_TYPES, "b_cat"), _stream(stream)), "salr_concat_adapters")


def salr_residual_adapter_workspace_bytes(N: int, K: int, r: int, oversample: int) -> int:
    return int(lib().salr_residual_adapter_workspace_bytes(N, K, r, oversample))


def salr_residual_adapter(e: torch.Tensor, r: int, oversample: int, power_iterations: int, omega: torch.Tensor,
                          a_res: torch.Tensor, b_res: torch.Tensor, sigma: Optional[torch.Tensor],
                          workspace: torch.Tensor, stream=None) -> None:
    """Enqueue the rank-r residual adapter of E [N, K]: a_res [K, r], b_res [r, N] (bf16), sigma [r] (fp32)."""
    N, K = e.shape
    if tuple(omega.shape) != (K, r + oversample) or omega.dtype != torch.float32 or not omega.is_contiguous():
        raise ValueError("omega must be a contiguous fp32 [K, r + oversample] tensor")
    if tuple(a_res.shape) != (K, r) or tuple(b_res.shape) != (r, N):
        raise ValueError("a_res must be [K, r] and b_res [r, N]")
    if sigma is not None and (sigma.dtype != torch.float32 or sigma.numel() != r):
        raise ValueError("sigma must hold r fp32 values")
    st = lib().salr_residual_adapter(_ptr(e, _BF16_TYPES, "e"), N, K, r, oversample, power_iterations,
                                     _ptr(omega, (torch.float32,), "omega"), _ptr(a_res, _BF16_TYPES, "a_res"),
                                     _ptr(b_res, _BF16_TYPES, "b_res"),
                                     None if sigma is None else _ptr(sigma, (torch.float32,), "sigma"),
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "salr_residual_adapter")


def residual_adapter(e: torch.Tensor, r: int, omega: torch.Tensor, power_iterations: int = 2):
    """(a_res, b_res, sigma) with oversample = omega.shape[1] - r."""
    N, K = e.shape
    oversample = omega.shape[1] - r
    need = salr_residual_adapter_workspace_bytes(N, K, r, oversample)
    if need == 0:
        raise ValueError("sizes not supported by salr_residual_adapter")
    ws = torch.empty(need, dtype=torch.uint8, device=e.device)
    a_res = torch.empty((K, r), dtype=e.dtype, device=e.device)
    b_res = torch.empty((r, N), dtype=e.dtype, device=e.device)
    sigma = torch.empty(r, dtype=torch.float32, device=e.device)
    salr_residual_adapter(e, r, oversample, power_iterations, omega, a_res, b_res, sigma, ws)
    return a_res, b_res, sigma


def residual(w: torch.Tensor, w_hat: torch.Tensor) -> torch.Tensor:
    e = torch.empty_like(w)
    salr_residual(w, w_hat, e)
    return e


def concat_adapters(a_list: Sequence[torch.Tensor], b_list: Sequence[torch.Tensor]) -> Tuple[torch.Tensor, torch.Tensor]:
    R = sum(a.shape[1] for a in a_list)
    a_cat = torch.empty((a_list[0].shape[0], R), dtype=a_list[0].dtype, device=a_list[0].device)
    b_cat = torch.empty((R, b_list[0].shape[1]), dtype=b_list[0].dtype, device=b_list[0].device)
    salr_concat_adapters(a_list, b_list, a_cat, b_cat)
    return a_cat, b_cat


def encode(w_dense: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """(bitmap, values, row_offsets) of an already pruned dense matrix; two passes with one sync
    in between to size ``values``."""
    rows, cols = w_dense.shape
    dev = w_dense.device
    bitmap = torch.empty((rows, salr_bitmap_words_per_row(cols)), dtype=torch.int32, device=dev)
    offsets = torch.empty(rows + 1, dtype=torch.int32, device=dev)
    salr_encode_bitmap(w_dense, bitmap, None, offsets)
    nnz = int(offsets[-1].item()) & 0xFFFFFFFF
    values = values_alloc(nnz, dev)
    salr_encode_bitmap(w_dense, bitmap, values, offsets)
    return bitmap, values, offsets


def decode(bitmap: torch.Tensor, values: torch.Tensor, row_offsets: torch.Tensor, rows: int, cols: int
           ) -> torch.Tensor:
    out = torch.empty((rows, cols), dtype=torch.int16, device=bitmap.device)
    salr_decode(bitmap, values, row_offsets, rows, cols, out)
    return out


def bitmap_is_2of4(bitmap: torch.Tensor) -> bool:
    """Check a layer once (synchronises): does every aligned group of four columns hold exactly two stored values?"""
    flag = torch.zeros(1, dtype=torch.int32, device=bitmap.device)
    salr_bitmap_is_2of4(bitmap, flag)
    return bool(int(flag.item()) == 1)


def linear_2of4(x, bitmap, values, row_offsets, a_cat, b_cat, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, K = x.shape
    N = bitmap.shape[0]
    R = 0 if a_cat is None else a_cat.shape[1]
    y = torch.empty((M, N), dtype=x.dtype, device=x.device)
    need = salr_linear_2of4_workspace_bytes(M, K, N, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    salr_sparse_lowrank_linear_2of4(x, bitmap, values, row_offsets, a_cat, b_cat, y, workspace)
    return y


def build_slice_table(bitmap, row_offsets, K: int) -> torch.Tensor:
    N = bitmap.shape[0]
    table = torch.empty((N, 8, 2), dtype=torch.int32, device=bitmap.device)
    salr_build_slice_table(bitmap, row_offsets, K, table)
    return table


def linear_prepared(x, bitmap, values, row_offsets, slice_table, a_cat, b_cat,
                    workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, K = x.shape
    N = bitmap.shape[0]
    R = 0 if a_cat is None else a_cat.shape[1]
    y = torch.empty((M, N), dtype=x.dtype, device=x.device)
    need = salr_linear_workspace_bytes(M, K, N, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    salr_sparse_lowrank_linear_prepared(x, bitmap, values, row_offsets, slice_table, a_cat, b_cat, y, workspace)
    return y


def linear(x, bitmap, values, row_offsets, a_cat, b_cat, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    M, K = x.shape
    N = bitmap.shape[0]
    R = 0 if a_cat is None else a_cat.shape[1]
    y = torch.empty((M, N), dtype=x.dtype, device=x.device)
    need = salr_linear_workspace_bytes(M, K, N, R)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    salr_sparse_lowrank_linear(x, bitmap, values, row_offsets, a_cat, b_cat, y, workspace)
    return y
