"""SALR CPU oracle -- TEST INFRASTRUCTURE, not part of the product.

Python face of ``oracle/salr_oracle.c`` (plain C, fp64) plus the few numpy-only checks that need an
SVD or the normal distribution.  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import this package; the HIP library and its binding never do, and this
package imports nothing from them.

All bf16 tensors are ``numpy.uint16`` arrays of raw bit patterns.  Orientation: W-hat is
``[N = out, K = in]`` (the transpose of the paper's ``W in R^{d_in x d_out}``), the bitmap is
``[N, ceil(K/32)]`` uint32 with bit t of word w = column ``32 w + t``.

Pins (see tests/test_oracle_*.py): the masks against a brute-force rank count (the N:M mask also against
the row mask applied to each group), the paper's printed
rule and Theorem 1's closed form and worked example; encode/decode against each other, the paper's
byte-mask/LUT decoder, popcount identities and hand-worked masks; the linear against pure-Python
loops, numpy fp64 matmul in the special cases that reduce to it, and the per-adapter sum; the SVD
residual against Theorem 3's bound; the residual against W = What + E and hand-worked values; the
concatenation against the sum over adapters on integer-valued matrices; the backward pass against the
forward pass (C code, not numpy) through the adjoint identities and against pure-Python loops; the NF4
quantiser of the packed values (QSALR) against a brute-force nearest-entry search in exact rational arithmetic,
hand-worked blocks, its error bound, idempotence and scale invariance, and the code book against the quantile
rule it comes from; the slice table (a derived index of the format) against pure-Python bit loops, the row offsets it
must start from and end at, and the popcounts of the decoded matrix.  No function here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import math
import os
from statistics import NormalDist
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsalr_oracle.so")
_lib = None

_u16p = ctypes.POINTER(ctypes.c_uint16)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_f64p = ctypes.POINTER(ctypes.c_double)
_i8p = ctypes.POINTER(ctypes.c_int8)
_i64 = ctypes.c_int64


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(
            os.path.join(_HERE, "salr_oracle.c")):
        from . import build as _build
        _build.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    lib.salr_oracle_threads.restype = ctypes.c_int
    lib.salr_oracle_words_per_row.restype = _i64
    lib.salr_oracle_words_per_row.argtypes = [_i64]
    lib.salr_oracle_mask_topk_rows.argtypes = [_u16p, _i64, _i64, _i64, _u16p]
    lib.salr_oracle_mask_threshold.argtypes = [_u16p, _i64, ctypes.c_uint16, _u16p]
    lib.salr_oracle_mask_nm.argtypes = [_u16p, _i64, _i64, _i64, _i64, _u16p]
    lib.salr_oracle_encode.argtypes = [_u16p, _i64, _i64, _u32p, _u16p, _i64, _u32p]
    lib.salr_oracle_decode.argtypes = [_u32p, _u16p, _u32p, _i64, _i64, _u16p]
    lib.salr_oracle_decode_lut.argtypes = [_u32p, _u16p, _u32p, _i64, _i64, _u16p]
    lib.salr_oracle_build_lut.argtypes = [_i8p]
    lib.salr_oracle_build_lut.restype = None
    lib.salr_oracle_linear.argtypes = [_u16p, _i64, _i64, _i64, _u16p, _u16p, _u16p, _i64, _f64p]
    lib.salr_oracle_adapter_accumulate.argtypes = [_u16p, _i64, _i64, _i64, _u16p, _u16p, _i64, _f64p]
    lib.salr_oracle_nf4_codebook.argtypes = [ctypes.POINTER(ctypes.c_float)]
    lib.salr_oracle_nf4_codebook.restype = None
    lib.salr_oracle_nf4_quantize.argtypes = [_u16p, _i64, ctypes.POINTER(ctypes.c_uint8), _u16p]
    lib.salr_oracle_nf4_dequantize.argtypes = [ctypes.POINTER(ctypes.c_uint8), _u16p, _i64, _u16p]
    _lib = lib
    return lib


def _p(a: Optional[np.ndarray], typ):
    if a is None:
        return ctypes.cast(None, typ)
    return a.ctypes.data_as(typ)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def threads() -> int:
    """Threads the OpenMP loops of the oracle use on this machine."""
    return int(_load().salr_oracle_threads())


def words_per_row(cols: int) -> int:
    return int(_load().salr_oracle_words_per_row(cols))


def mask_topk_rows(w: np.ndarray, keep: int) -> np.ndarray:
    """Per-row magnitude pruning (Sec. 2): keep the ``keep`` largest |w| of every row, ties to the
    lower column, +0.0 elsewhere."""
    w = _c(w, np.uint16)
    rows, cols = w.shape
    out = np.empty_like(w)
    rc = _load().salr_oracle_mask_topk_rows(_p(w, _u16p), rows, cols, int(keep), _p(out, _u16p))
    if rc:
        raise RuntimeError(f"mask_topk_rows failed ({rc})")
    return out


def mask_threshold(w: np.ndarray, t_mag: int) -> np.ndarray:
    """The rule as printed in Sec. 2: keep iff |w| > T for one threshold magnitude (bf16 pattern)."""
    w = _c(w, np.uint16)
    out = np.empty_like(w)
    rc = _load().salr_oracle_mask_threshold(_p(w, _u16p), w.size, int(t_mag), _p(out, _u16p))
    if rc:
        raise RuntimeError("mask_threshold failed")
    return out


def mask_nm(w: np.ndarray, n_keep: int, m_group: int) -> np.ndarray:
    """N:M pruning (Sec. 4, the 2:4 pattern of the inference table): keep the n largest |w| of every m
    consecutive columns, ties to the lower column."""
    w = _c(w, np.uint16)
    rows, cols = w.shape
    out = np.empty_like(w)
    rc = _load().salr_oracle_mask_nm(_p(w, _u16p), rows, cols, int(n_keep), int(m_group), _p(out, _u16p))
    if rc:
        raise RuntimeError(f"mask_nm failed ({rc})")
    return out


def encode(w_hat: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Bitmap + packed nonzeros + row offsets of a dense (already pruned) matrix (Sec. 3.3)."""
    w_hat = _c(w_hat, np.uint16)
    rows, cols = w_hat.shape
    wpr = words_per_row(cols)
    bitmap = np.empty((rows, wpr), dtype=np.uint32)
    offsets = np.empty(rows + 1, dtype=np.uint32)
    lib = _load()
    rc = lib.salr_oracle_encode(_p(w_hat, _u16p), rows, cols, _p(bitmap, _u32p), _p(None, _u16p), 0,
                                _p(offsets, _u32p))
    if rc:
        raise RuntimeError(f"encode (count) failed ({rc})")
    nnz = int(offsets[rows])
    values = np.empty(nnz, dtype=np.uint16)
    rc = lib.salr_oracle_encode(_p(w_hat, _u16p), rows, cols, _p(bitmap, _u32p), _p(values, _u16p), nnz,
                                _p(offsets, _u32p))
    if rc:
        raise RuntimeError(f"encode failed ({rc})")
    return bitmap, values, offsets


def decode(bitmap: np.ndarray, values: np.ndarray, row_offsets: np.ndarray, rows: int, cols: int,
           use_lut: bool = False) -> np.ndarray:
    """Dense matrix back from the format.  ``use_lut`` selects the paper's byte-mask + lookup-table
    decoder instead of the running-cursor one."""
    bitmap = _c(bitmap, np.uint32)
    values = _c(values, np.uint16)
    row_offsets = _c(row_offsets, np.uint32)
    out = np.empty((rows, cols), dtype=np.uint16)
    fn = _load().salr_oracle_decode_lut if use_lut else _load().salr_oracle_decode
    rc = fn(_p(bitmap, _u32p), _p(values, _u16p), _p(row_offsets, _u32p), rows, cols, _p(out, _u16p))
    if rc:
        raise RuntimeError(f"decode failed ({rc})")
    return out


def slice_table(bitmap: np.ndarray, row_offsets: np.ndarray, cols: int, slices: int = 8) -> np.ndarray:
    """Where the packed values of a range of columns start (Sec. 3.3: the value array is read sequentially, so the
    position of a column's value is the number of set bits before it).  For row n and slice w of the row's
    C = ceil(cols / 128) chunks of 128 columns, slice w = chunks [C w / slices, C (w + 1) / slices):
        out[n, w, 0] = row_offsets[n] + set bits of row n in the columns before the slice
        out[n, w, 1] = the most set bits that any one chunk of the slice holds.
    Written out on the bit matrix itself, column by column range."""
    bitmap = _c(bitmap, np.uint32)
    row_offsets = _c(row_offsets, np.uint32)
    rows = bitmap.shape[0]
    bits = np.unpackbits(bitmap.view(np.uint8).reshape(rows, -1), axis=1, bitorder="little")[:, :cols].astype(np.int64)
    chunks = (cols + 127) // 128
    out = np.zeros((rows, slices, 2), dtype=np.uint32)
    for w in range(slices):
        c0, c1 = chunks * w // slices, chunks * (w + 1) // slices
        before = bits[:, :min(128 * c0, cols)].sum(axis=1)
        out[:, w, 0] = (row_offsets[:rows].astype(np.int64) + before).astype(np.uint32)
        longest = np.zeros(rows, dtype=np.int64)
        for c in range(c0, c1):
            longest = np.maximum(longest, bits[:, 128 * c:min(128 * (c + 1), cols)].sum(axis=1))
        out[:, w, 1] = longest.astype(np.uint32)
    return out


def build_lut() -> np.ndarray:
    """The 256 x 8 table of Sec. 3.3: entry [m, t] = index of bit t among m's set bits, or -1."""
    lut = np.empty((256, 8), dtype=np.int8)
    _load().salr_oracle_build_lut(_p(lut, _i8p))
    return lut


def linear(x: np.ndarray, w_hat: np.ndarray, a_cat: Optional[np.ndarray], b_cat: Optional[np.ndarray]
           ) -> np.ndarray:
    """Y = X What^T + (X A_cat) B_cat in fp64 (Sec. 3.2).  ``a_cat``/``b_cat`` None means R = 0."""
    x = _c(x, np.uint16)
    w_hat = _c(w_hat, np.uint16)
    M, K = x.shape
    N, K2 = w_hat.shape
    if K != K2:
        raise ValueError("K mismatch")
    R = 0
    if a_cat is not None:
        a_cat = _c(a_cat, np.uint16)
        b_cat = _c(b_cat, np.uint16)
        R = a_cat.shape[1]
        if a_cat.shape != (K, R) or b_cat.shape != (R, N):
            raise ValueError("adapter shapes")
    y = np.empty((M, N), dtype=np.float64)
    rc = _load().salr_oracle_linear(_p(x, _u16p), M, K, N, _p(w_hat, _u16p),
                                    _p(a_cat if R else None, _u16p), _p(b_cat if R else None, _u16p), R,
                                    _p(y, _f64p))
    if rc:
        raise RuntimeError(f"linear failed ({rc})")
    return y


def linear_per_adapter(x: np.ndarray, w_hat: np.ndarray, As: Sequence[np.ndarray],
                       Bs: Sequence[np.ndarray]) -> np.ndarray:
    """y = x What^T + sum_i (x A_i) B_i, one adapter at a time (Sec. 3.2 before concatenation)."""
    y = linear(x, w_hat, None, None)
    x = _c(x, np.uint16)
    M, K = x.shape
    N = w_hat.shape[0]
    for a, b in zip(As, Bs):
        a = _c(a, np.uint16)
        b = _c(b, np.uint16)
        r = a.shape[1]
        rc = _load().salr_oracle_adapter_accumulate(_p(x, _u16p), M, K, N, _p(a, _u16p), _p(b, _u16p), r,
                                                    _p(y, _f64p))
        if rc:
            raise RuntimeError("adapter_accumulate failed")
    return y


def linear_backward(x: np.ndarray, dy: np.ndarray, w_hat: np.ndarray, a_cat: Optional[np.ndarray],
                    b_cat: Optional[np.ndarray]) -> Tuple[np.ndarray, Optional[np.ndarray], Optional[np.ndarray]]:
    """The adjoint of the layer Y = X What^T + (X A_cat) B_cat (Sec. 3.2 / 3.3) in fp64, written out from the chain
    rule: dX = dY What + (dY B_cat^T) A_cat^T, dA = X^T (dY B_cat^T), dB = (X A_cat)^T dY.  bf16 patterns in, fp64 out.
    The frozen What gets no gradient."""
    X, dY, W = bf16_to_f64(x), bf16_to_f64(dy), bf16_to_f64(w_hat)
    dX = dY @ W
    if a_cat is None or a_cat.shape[1] == 0:
        return dX, None, None
    A, B = bf16_to_f64(a_cat), bf16_to_f64(b_cat)
    Tp = dY @ B.T            # [M, R]
    return dX + Tp @ A.T, X.T @ Tp, (X @ A).T @ dY


# ---------------------------------------------------------------------------------------------------
# numpy-only checks of the paper's closed forms
# ---------------------------------------------------------------------------------------------------

def pruning_mse_closed_form(p: float, sigma: float = 1.0) -> float:
    """Theorem 1: MSE(p) = 2 sigma^2 [Phi(t_p) - 1/2 - t_p phi(t_p)], t_p = Phi^{-1}((1+p)/2)."""
    nd = NormalDist()
    t = nd.inv_cdf((1.0 + p) / 2.0)
    phi = math.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)
    return 2.0 * sigma * sigma * (nd.cdf(t) - 0.5 - t * phi)


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 bit patterns, nearest even (NaN stays NaN).  Written out on the integer patterns:
    add 0x7FFF plus the lowest kept bit, drop the low 16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    rounded = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)
    nan = (u & np.uint64(0x7FFFFFFF)) > np.uint64(0x7F800000)
    return np.where(nan, (u >> np.uint64(16)) | np.uint64(0x40), rounded).astype(np.uint16)


def residual(w: np.ndarray, w_hat: np.ndarray) -> np.ndarray:
    """Sec. 3.1: E = W - What, entry by entry; the subtraction in fp32 (exact whenever What is a masked W),
    the result as bf16 patterns."""
    a = (np.ascontiguousarray(w, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    b = (np.ascontiguousarray(w_hat, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    with np.errstate(invalid="ignore", over="ignore"):   # Inf - Inf and NaN operands are legal inputs
        return f32_to_bf16(a - b)


def concat_adapters(As: Sequence[np.ndarray], Bs: Sequence[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Sec. 3.2: A_cat = [A_1 ... A_n] in R^{d_in x (sum r_i)}, B_cat = [B_1; ...; B_n] in R^{(sum r_i) x d_out}."""
    K, N = As[0].shape[0], Bs[0].shape[1]
    R = sum(a.shape[1] for a in As)
    a_cat = np.zeros((K, R), dtype=As[0].dtype)
    b_cat = np.zeros((R, N), dtype=Bs[0].dtype)
    first = 0
    for a, b in zip(As, Bs):
        r = a.shape[1]
        assert a.shape == (K, r) and b.shape == (r, N)
        for c in range(r):
            a_cat[:, first + c] = a[:, c]
            b_cat[first + c, :] = b[c, :]
        first += r
    return a_cat, b_cat


def svd_residual_check(w: np.ndarray, w_hat: np.ndarray, r: int) -> Tuple[float, float]:
    """Sec. 3.1 / Theorem 3: E = W - What, E_r = rank-r truncated SVD of E.
    Returns (||E||_F^2 / (N K),  ||E - E_r||_F^2 / ||E||_F^2)."""
    E = bf16_to_f64(w) - bf16_to_f64(w_hat)
    s = np.linalg.svd(E, compute_uv=False)
    total = float(np.sum(s * s))
    tail = float(np.sum(s[r:] ** 2))
    return total / E.size, (tail / total if total > 0 else 0.0)


def svd_residual_adapter(w: np.ndarray, w_hat: np.ndarray, r: int) -> Tuple[np.ndarray, np.ndarray]:
    """The residual adapter of Sec. 3.1 in our orientation, fp64: with E = U S V^T ([N, K]),
    A = V_r S_r^{1/2} ([K, r]) and B = S_r^{1/2} U_r^T ([r, N]) so that A B = E_r^T."""
    E = bf16_to_f64(w) - bf16_to_f64(w_hat)
    U, s, Vt = np.linalg.svd(E, full_matrices=False)
    rs = np.sqrt(s[:r])
    return Vt[:r].T * rs[None, :], (U[:, :r] * rs[None, :]).T


def nf4_codebook() -> np.ndarray:
    """The 16 NF4 levels (fp32), ascending, as the oracle uses them."""
    out = np.empty(16, dtype=np.float32)
    _load().salr_oracle_nf4_codebook(out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    return out


def nf4_quantize(values: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """QSALR (Sec. 4): packed bf16 values -> (codes uint8 [ceil(n/2)], two 4-bit codes per byte, even index in the low
    nibble; scales bf16 bits [ceil(n/64)], one per block of 64 consecutive values)."""
    v = _c(np.asarray(values).reshape(-1), np.uint16)
    n = v.size
    codes = np.zeros((n + 1) // 2, dtype=np.uint8)
    scales = np.zeros((n + 63) // 64, dtype=np.uint16)
    rc = _load().salr_oracle_nf4_quantize(_p(v, _u16p), n, codes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                          _p(scales, _u16p))
    if rc:
        raise RuntimeError(f"nf4_quantize failed ({rc})")
    return codes, scales


def nf4_dequantize(codes: np.ndarray, scales: np.ndarray, count: int) -> np.ndarray:
    """The bf16 values the codes stand for: bf16(level[code] * scale of the block), the product in fp32."""
    c = _c(codes, np.uint8)
    sc = _c(scales, np.uint16)
    if c.size < (count + 1) // 2 or sc.size < (count + 63) // 64:
        raise ValueError("codes / scales too short")
    out = np.zeros(count, dtype=np.uint16)
    rc = _load().salr_oracle_nf4_dequantize(c.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), _p(sc, _u16p), count,
                                            _p(out, _u16p))
    if rc:
        raise RuntimeError(f"nf4_dequantize failed ({rc})")
    return out
