"""The C-ABI library loads, exports every symbol include/salr.h declares, and validates arguments on
the host before any launch.  No GPU needed: no call here reaches a kernel."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "salr.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(salr_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2601_16991_amd as salr
    if not os.path.exists(salr.LIB_PATH):
        from paper_2601_16991_amd import build
        build.build()
    return salr.lib()


def test_header_declares_the_three_operations():
    names = _declared_functions()
    for required in ("salr_encode_bitmap", "salr_decode", "salr_sparse_lowrank_linear"):
        assert required in names


def test_every_declared_symbol_is_exported(lib):
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_status_strings(lib):
    seen = set()
    for code in range(6):
        s = lib.salr_status_string(code)
        assert s and s not in seen
        seen.add(s)


def test_words_per_row(lib):
    assert lib.salr_bitmap_words_per_row(0) == 0
    assert lib.salr_bitmap_words_per_row(1) == 1
    assert lib.salr_bitmap_words_per_row(32) == 1
    assert lib.salr_bitmap_words_per_row(33) == 2
    assert lib.salr_bitmap_words_per_row(14336) == 448
    assert lib.salr_bitmap_words_per_row(-1) == -1


def _r256(b):
    return (b + 255) // 256 * 256


def _t_ksplit(M, K):
    rows = 256 if M >= 4096 else 64
    blocks, units, s = (M + rows - 1) // rows, K // 32, 1
    while s < 64 and blocks * s * 2 <= 1024 and units // (s * 2) >= 8:
        s *= 2
    return s


def _y_ksplit(M, K, N):
    tiles, steps, s = ((M + 255) // 256) * ((N + 127) // 128), K // 64, 1
    if tiles >= 128 or N % 4:
        return 1
    while s < 8 and tiles * s * 2 <= 256 and steps % (s * 2) == 0 and steps // (s * 2) >= 4:
        s *= 2
    return s


def _rowtile(M, K, N):
    """Batches of 9..128 tokens on whole 128-column chunks take the row-tiled streaming path (from 33 tokens on, or on
    layers of 8192 rows and more); not when K cannot be split (N % 4) and the 128-row tiles are few."""
    if M > 128 or K < 128 or K % 128:
        return False
    if N % 4 and N < 64 * 128:
        return False
    return M > 32 or (M > 8 and N >= 8192)


def _rowtile_ksplit(M, K, N):
    tiles, chunks, s = (N + 127) // 128, K // 128, 1
    if N % 4:
        return 1
    while s < 16 and tiles * s < (448 if M <= 64 else 224) and chunks // (s * 2) >= 4:
        s *= 2
    return s


def _own_table(M, K, N, R):
    """A call with adapters whose kernel starts from cursors keeps a slice table of its own (64 bytes per weight row)
    behind the rest: rows of whole chunks, up to 64 tokens (not the long-row kernel's shapes), or the row-tiled kernel with K split 1, 2, 4 or 8 ways."""
    if R <= 0 or K < 128 or K % 128:
        return 0
    if _rowtile(M, K, N):
        return _r256(64 * N) if 8 % _rowtile_ksplit(M, K, N) == 0 else 0
    if M <= 16 and 12288 <= K <= 32768:   # the long-row kernel: reads a caller's table, builds none
        return 0
    return _r256(64 * N) if M <= 64 else 0


def _expected_workspace(M, K, N, R):
    """The documented layout, restated.  Row-tiled path: sixteen fp32 split-K partials of T, then fp32 split-K
    partials of Y when K is split.  Else M <= 64: sixteen fp32 split-K partials of T.  Larger M: T [M, Rpad] bf16,
    transposed padded A_cat [Rpad, K] bf16, fp32 split-K partials of T; for K % 64 == 0 also the decoded weight [N, K]
    bf16 and, when the output has few tiles, fp32 split-K partials of Y.  Each part rounded to 256 B.  Last, the call's
    own slice table where it keeps one."""
    rp = (R + 31) // 32 * 32
    if _rowtile(M, K, N):
        ks = _rowtile_ksplit(M, K, N)
        return (_r256(16 * M * rp * 4) if R else 0) + (_r256(ks * M * N * 4) if ks > 1 else 0) + _own_table(M, K, N, R)
    if M <= 64:
        return (_r256(16 * M * rp * 4) if R else 0) + _own_table(M, K, N, R)
    b = 0
    if R:
        b += _r256(M * rp * 2) + _r256(K * rp * 2)
        ks = 16 if M <= 1024 else _t_ksplit(M, K)   # up to 1024 rows: the sixteen partials of the small-batch pre-kernel
        if ks > 1:
            b += _r256(ks * M * rp * 4)
    if K >= 64 and K % 64 == 0:
        b += _r256(N * K * 2)
        ks = _y_ksplit(M, K, N)
        if ks > 1:
            b += _r256(ks * M * N * 4)
    return b


def test_workspace_bytes(lib):
    assert lib.salr_linear_workspace_bytes(16, 4096, 4096, 0) == 0
    assert lib.salr_linear_workspace_bytes(0, 4096, 4096, 32) == 0
    assert lib.salr_linear_workspace_bytes(16, 4096, 4096, 32) == 16 * 16 * 32 * 4 + 64 * 4096   # T partials + slice table
    assert lib.salr_linear_workspace_bytes(1, 4096, 4096, 64) == 16 * 64 * 4 + 64 * 4096
    assert lib.salr_linear_workspace_bytes(16, 4000, 4096, 32) == 16 * 16 * 32 * 4               # ragged rows: no table
    assert lib.salr_linear_workspace_bytes(32, 4096, 4096, 0) == 0
    assert lib.salr_linear_workspace_bytes(128, 4096, 28672, 0) == 0           # 224 row tiles: K is not split
    assert lib.salr_linear_workspace_bytes(64, 4096, 28672, 0) == 2 * 64 * 28672 * 4   # up to 64 tokens: 448 workgroups wanted
    assert lib.salr_linear_workspace_bytes(64, 4096, 20480, 0) == 4 * 64 * 20480 * 4   # 160 row tiles, up to 64 tokens: 448 workgroups wanted
    assert lib.salr_linear_workspace_bytes(64, 4096, 4096, 0) == 8 * 64 * 4096 * 4     # 32 row tiles: K split 8 ways (4 chunks each)
    assert lib.salr_linear_workspace_bytes(24, 4096, 8192, 16) == 16 * 24 * 32 * 4 + 8 * 24 * 8192 * 4 + 64 * 8192   # 64 row tiles: K split 8 ways
    assert lib.salr_linear_workspace_bytes(128, 4000, 4096, 0) == 0            # K % 64 != 0: no dense scratch
    assert lib.salr_linear_workspace_bytes(16, 4096, 4096, 1000) == 0          # rank not supported
    assert lib.salr_linear_workspace_bytes(2048, 4096, 14336, 0) == 14336 * 4096 * 2
    assert _t_ksplit(4096, 14336) == 32 and _t_ksplit(2048, 4096) == 16 and _y_ksplit(512, 14336, 4096) == 4
    for (M, K, N, R) in [(16, 4096, 4096, 16), (65, 4096, 4096, 1), (128, 4096, 4096, 32), (255, 64, 8, 7),
                         (33, 14336, 4096, 64), (100, 128, 130, 3), (129, 4096, 4096, 32), (64, 4096, 28672, 40),
                         (20, 1024, 8192, 8), (20, 1024, 8190, 8), (70, 4000, 4096, 8), (9, 1024, 8192, 8), (8, 1024, 8192, 8),
                         (16, 4096, 28672, 32), (40, 1152, 28672, 32), (100, 4096, 28672, 32),
                         (256, 4096, 4096, 0), (256, 4096, 4096, 32), (512, 14336, 4096, 64), (2048, 4096, 14336, 32),
                         (4096, 14336, 4096, 64), (8, 14336, 4096, 64), (1, 28672, 8192, 64), (16, 12160, 512, 8), (1024, 96, 8, 32), (1024, 64, 8, 0), (300, 1024, 262, 5)]:
        assert lib.salr_linear_workspace_bytes(M, K, N, R) == _expected_workspace(M, K, N, R), (M, K, N, R)


def test_host_validation_rejects_before_launch(lib):
    import paper_2601_16991_amd as salr
    fake = 0x1000  # never dereferenced: every call below fails validation first
    # negative sizes
    assert lib.salr_encode_bitmap(fake, -1, 8, fake, None, 0, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_decode(fake, fake, fake, 4, -2, fake, None) == salr.SALR_ERR_INVALID_ARG
    # null pointers
    assert lib.salr_encode_bitmap(None, 4, 8, fake, None, 0, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_encode_bitmap(fake, 4, 8, fake, None, 0, None, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_decode(None, fake, fake, 4, 8, fake, None) == salr.SALR_ERR_INVALID_ARG
    # nnz would not fit 32 bits
    assert lib.salr_encode_bitmap(fake, 1 << 20, 1 << 20, fake, None, 0, fake, None) == salr.SALR_ERR_SHAPE
    # linear: K not a multiple of 32, rank too large, workspace missing / too small, null adapters
    args = dict(M=4, K=64, N=8, R=4)

    def lin(M=4, K=64, N=8, R=4, x=fake, a=fake, b=fake, ws=fake, ws_bytes=1 << 20, y=fake):
        return lib.salr_sparse_lowrank_linear(x, M, K, N, fake, fake, fake, a, b, R, y, ws, ws_bytes, None)

    assert lin(K=40) == salr.SALR_ERR_SHAPE
    assert lin(R=257) == salr.SALR_ERR_UNSUPPORTED
    assert lin(ws=None) == salr.SALR_ERR_CAPACITY
    assert lin(ws_bytes=16) == salr.SALR_ERR_CAPACITY
    assert lin(a=None) == salr.SALR_ERR_INVALID_ARG
    assert lin(x=None) == salr.SALR_ERR_INVALID_ARG
    assert lin(y=None) == salr.SALR_ERR_INVALID_ARG
    assert lin(M=-1) == salr.SALR_ERR_INVALID_ARG
    # empty problems are no-ops
    assert lin(M=0) == salr.SALR_OK
    assert lin(N=0) == salr.SALR_OK
    # an empty contraction (K == 0) is legal with null x / bitmap / values / adapters: it passes validation (what
    # follows is one fill of Y with zeros, which needs a device: without one the launch reports SALR_ERR_HIP)
    st = lib.salr_sparse_lowrank_linear(None, 4, 0, 8, None, None, None, None, None, 4, fake, None, 0, None)
    assert st in (salr.SALR_OK, salr.SALR_ERR_HIP)
    assert lib.salr_sparse_lowrank_linear(None, 4, 0, 8, None, None, None, None, None, 4, None, None, 0, None) \
        == salr.SALR_ERR_INVALID_ARG     # Y is still required
    # masks: keep outside [0, cols], group sizes, null pointers, empty inputs
    assert lib.salr_magnitude_mask_rows(fake, 4, 8, 9, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_magnitude_mask_rows(fake, 4, 8, -1, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_magnitude_mask_rows(None, 4, 8, 4, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_magnitude_mask_rows(fake, 0, 8, 4, fake, None) == salr.SALR_OK
    assert lib.salr_magnitude_mask_nm(fake, 4, 8, 3, 2, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_magnitude_mask_nm(fake, 4, 8, 1, 0, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_magnitude_mask_nm(fake, 4, 10, 2, 4, fake, None) == salr.SALR_ERR_SHAPE
    assert lib.salr_magnitude_mask_nm(fake, 4, 128, 2, 128, fake, None) == salr.SALR_ERR_UNSUPPORTED
    assert lib.salr_magnitude_mask_nm(fake, 4, 8, 2, 4, None, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_magnitude_mask_nm(fake, 0, 8, 2, 4, fake, None) == salr.SALR_OK


def test_residual_adapter_validation_and_workspace(lib):
    import paper_2601_16991_amd as salr
    fake = 0x1000  # never dereferenced: every call below fails validation first
    q = lib.salr_residual_adapter_workspace_bytes
    assert q(4096, 4096, 32, 16) > 4096 * 4096 * 2          # holds at least the transposed copy of E
    assert q(4096, 4096, 32, 16) % 256 == 0
    assert q(4096, 4100, 32, 16) == 0 and q(4096, 4096, 120, 16) == 0 and q(64, 64, 60, 8) == 0 and q(0, 64, 4, 4) == 0

    def call(N=64, K=96, r=8, over=8, iters=1, e=fake, omega=fake, a=fake, b=fake, ws=fake, ws_bytes=1 << 30):
        return lib.salr_residual_adapter(e, N, K, r, over, iters, omega, a, b, None, ws, ws_bytes, None)

    assert call(N=-1) == salr.SALR_ERR_INVALID_ARG
    assert call(e=None) == salr.SALR_ERR_INVALID_ARG
    assert call(omega=None) == salr.SALR_ERR_INVALID_ARG
    assert call(K=100) == salr.SALR_ERR_SHAPE
    assert call(r=60, over=8) == salr.SALR_ERR_SHAPE            # more sketch columns than min(N, K)
    assert call(N=256, K=256, r=120, over=16) == salr.SALR_ERR_UNSUPPORTED
    assert call(iters=65) == salr.SALR_ERR_UNSUPPORTED
    assert call(ws=None) == salr.SALR_ERR_CAPACITY
    assert call(ws_bytes=1024) == salr.SALR_ERR_CAPACITY
    assert call(r=0) == salr.SALR_OK and call(N=0) == salr.SALR_OK   # nothing to do


def test_residual_and_concat_validation(lib):
    import ctypes
    import paper_2601_16991_amd as salr
    fake = 0x1000
    assert lib.salr_residual(fake, fake, -1, 4, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_residual(None, fake, 4, 4, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_residual(None, None, 0, 4, None, None) == salr.SALR_OK
    ptrs = (ctypes.c_void_p * 2)(fake, fake)
    nulls = (ctypes.c_void_p * 2)(fake, None)
    ranks = (ctypes.c_int64 * 2)(4, 4)
    bad = (ctypes.c_int64 * 2)(4, -1)
    big = (ctypes.c_int64 * 2)(40000, 40000)
    assert lib.salr_concat_adapters(ptrs, ptrs, bad, 2, 8, 8, fake, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_concat_adapters(nulls, ptrs, ranks, 2, 8, 8, fake, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_concat_adapters(ptrs, ptrs, ranks, 2, 8, 8, None, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_concat_adapters(ptrs, ptrs, big, 2, 8, 8, fake, fake, None) == salr.SALR_ERR_SHAPE
    assert lib.salr_concat_adapters(None, None, None, 0, 8, 8, None, None, None) == salr.SALR_OK


def test_backward_validation_and_workspace(lib):
    import paper_2601_16991_amd as salr
    fake = 0x1000
    q = lib.salr_linear_backward_workspace_bytes
    assert q(512, 4096, 4096, 32, 1, 1) > 2 * 4096 * 4096 * 2     # decoded weight and its transpose
    assert q(512, 4096, 4096, 32, 0, 1) < q(512, 4096, 4096, 32, 1, 1)
    assert q(512, 4096, 4096, 32, 1, 1) % 256 == 0
    assert q(500, 4096, 4096, 32, 1, 1) == 0 and q(500, 4096, 4096, 32, 1, 0) > 0    # dA / dB want M % 32 == 0
    assert q(512, 4096, 4000, 32, 1, 0) == 0 and q(512, 4100, 4096, 32, 1, 0) == 0 and q(512, 4096, 4096, 300, 1, 1) == 0

    def call(M=64, K=64, N=64, R=8, x=fake, dy=fake, bm=fake, ro=fake, a=fake, b=fake, dx=fake, da=fake, db=fake, ws=fake,
             ws_bytes=1 << 30):
        return lib.salr_sparse_lowrank_linear_backward(x, dy, M, K, N, bm, fake, ro, a, b, R, dx, da, db, ws, ws_bytes, None)

    assert call(M=-1) == salr.SALR_ERR_INVALID_ARG
    assert call(dy=None) == salr.SALR_ERR_INVALID_ARG
    assert call(bm=None) == salr.SALR_ERR_INVALID_ARG
    assert call(x=None) == salr.SALR_ERR_INVALID_ARG              # dA / dB asked for
    assert call(a=None) == salr.SALR_ERR_INVALID_ARG
    assert call(K=40) == salr.SALR_ERR_SHAPE
    assert call(N=96) == salr.SALR_ERR_UNSUPPORTED                # dX wants N % 64 == 0
    assert call(M=40) == salr.SALR_ERR_UNSUPPORTED                # dA / dB want M % 32 == 0
    assert call(R=257) == salr.SALR_ERR_UNSUPPORTED
    assert call(ws=None) == salr.SALR_ERR_CAPACITY
    assert call(ws_bytes=64) == salr.SALR_ERR_CAPACITY
    assert call(dx=None, da=None, db=None) == salr.SALR_OK        # nothing asked for
    assert call(M=0) == salr.SALR_OK


def test_two_of_four_validation_and_workspace(lib):
    import ctypes
    import paper_2601_16991_amd as salr
    fake = 0x1000
    q, g = lib.salr_linear_2of4_workspace_bytes, lib.salr_linear_workspace_bytes
    q.restype = g.restype = ctypes.c_size_t
    # shapes the sparse-MFMA kernels take: the row-tiled layout (16 partials of T, partials of Y where K is split),
    # never less than the general call needs
    assert q(16, 4096, 4096, 32) == max(_r256(16 * 16 * 32 * 4) + _r256(8 * 16 * 4096 * 4), g(16, 4096, 4096, 32))
    assert q(128, 4096, 28672, 0) == g(128, 4096, 28672, 0) == 0
    assert q(1, 8192, 28672, 64) >= _r256(16 * 1 * 64 * 4)
    # shapes passed on to the general call: its workspace
    for (M, K, N, R) in [(200, 4096, 4096, 32), (16, 96, 64, 8), (2048, 4096, 14336, 32), (20, 640, 130, 8)]:
        assert q(M, K, N, R) == g(M, K, N, R), (M, K, N, R)
    assert q(16, 4096, 4096, 1000) == 0 and q(0, 4096, 4096, 8) == 0

    def call(M=16, K=256, N=64, R=8, x=fake, bm=fake, v=fake, ro=fake, a=fake, b=fake, y=fake, ws=fake, ws_bytes=1 << 30):
        return lib.salr_sparse_lowrank_linear_2of4(x, M, K, N, bm, v, ro, a, b, R, y, ws, ws_bytes, None)

    assert call(M=-1) == salr.SALR_ERR_INVALID_ARG
    assert call(x=None) == salr.SALR_ERR_INVALID_ARG
    assert call(bm=None) == salr.SALR_ERR_INVALID_ARG
    assert call(v=None) == salr.SALR_ERR_INVALID_ARG
    assert call(ro=None) == salr.SALR_ERR_INVALID_ARG
    assert call(y=None) == salr.SALR_ERR_INVALID_ARG
    assert call(a=None) == salr.SALR_ERR_INVALID_ARG
    assert call(K=40) == salr.SALR_ERR_SHAPE
    assert call(R=257) == salr.SALR_ERR_UNSUPPORTED
    assert call(ws=None) == salr.SALR_ERR_CAPACITY
    assert call(ws_bytes=64) == salr.SALR_ERR_CAPACITY
    assert call(M=0) == salr.SALR_OK
    assert call(M=200, y=None) == salr.SALR_ERR_INVALID_ARG       # passed on to the general call, which validates too

    chk = lib.salr_bitmap_is_2of4
    assert chk(fake, -1, 64, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert chk(fake, 4, 64, None, None) == salr.SALR_ERR_INVALID_ARG
    assert chk(None, 4, 64, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert chk(fake, 4, 40, fake, None) == salr.SALR_ERR_SHAPE


def test_qsalr_and_noalloc_validation(lib):
    import ctypes
    import paper_2601_16991_amd as salr
    fake = 0x1000   # never dereferenced: every call below fails validation first (or has nothing to do)
    assert lib.salr_nf4_quantize_values(fake, -1, fake, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_nf4_quantize_values(None, 8, fake, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_nf4_quantize_values(fake, 8, None, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_nf4_quantize_values(fake, 1 << 33, fake, fake, None) == salr.SALR_ERR_SHAPE
    assert lib.salr_nf4_quantize_values(None, 0, None, None, None) == salr.SALR_OK
    assert lib.salr_nf4_dequantize_values(fake, fake, -2, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_nf4_dequantize_values(fake, None, 8, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert lib.salr_nf4_dequantize_values(None, None, 0, None, None) == salr.SALR_OK
    q = lib.salr_qsalr_linear_workspace_bytes
    q.restype = ctypes.c_size_t
    g = lib.salr_linear_workspace_bytes
    # larger batches: the dequantised values (2 bytes each, whole 16-byte vectors, 256-byte aligned) in front of the
    # layer's own workspace
    assert q(65, 4096, 4096, 32, 1000) == _r256(2 * 1000) + g(65, 4096, 4096, 32)
    assert q(65, 4096, 4096, 32, 1001) == _r256(2 * 1008) + g(65, 4096, 4096, 32)
    assert q(16, 4128, 4096, 32, 1000) == _r256(2 * 1000) + g(16, 4128, 4096, 32)    # rows that are not whole chunks
    # large batches on rows of whole 64-column steps: the decode stage reads the codes, the workspace is the plain layer's
    assert q(2048, 4096, 4096, 32, 10 ** 6) == g(2048, 4096, 4096, 32)
    assert q(300, 4128, 4096, 32, 1000) == _r256(2 * 1000) + g(300, 4128, 4096, 32)   # K % 64 != 0: dequantise first
    # up to 64 tokens on rows of whole 128-column chunks: no bf16 copy of the values, only the sixteen fp32 partials
    # of T and the call's slice table (64 bytes per weight row)
    assert q(16, 4096, 4096, 32, 1000) == 16 * 16 * 32 * 4 + 64 * 4096
    assert q(64, 4096, 14336, 0, 10 ** 7) == 64 * 14336
    assert q(1, 128, 3, 5, 7) == _r256(16 * 1 * 32 * 4) + _r256(64 * 3)
    assert q(16, 4096, 4096, 32, 0) == g(16, 4096, 4096, 32)       # no stored values: the plain layer
    assert q(16, 4100, 4096, 32, 1000) == 0 and q(16, 4096, 4096, 32, -1) == 0

    def call(M=4, K=64, N=8, R=4, nnz=100, x=fake, codes=fake, scales=fake, y=fake, ws=fake, ws_bytes=1 << 20):
        return lib.salr_qsalr_linear(x, M, K, N, fake, codes, scales, fake, nnz, fake, fake, R, y, ws, ws_bytes, None)

    assert call(nnz=-1) == salr.SALR_ERR_INVALID_ARG
    assert call(codes=None) == salr.SALR_ERR_INVALID_ARG
    assert call(scales=None) == salr.SALR_ERR_INVALID_ARG
    assert call(K=40) == salr.SALR_ERR_SHAPE
    assert call(nnz=4 * 64 * 8) == salr.SALR_ERR_SHAPE          # more stored values than the matrix has elements
    assert call(R=300) == salr.SALR_ERR_UNSUPPORTED
    assert call(ws=None) == salr.SALR_ERR_CAPACITY
    assert call(ws_bytes=128) == salr.SALR_ERR_CAPACITY
    assert call(M=0) == salr.SALR_OK
    # the small-batch kernel's shapes (K a multiple of 128, up to 64 tokens) validate the same way
    assert call(K=128, nnz=-1) == salr.SALR_ERR_INVALID_ARG
    assert call(K=128, codes=None) == salr.SALR_ERR_INVALID_ARG
    assert call(K=128, x=None) == salr.SALR_ERR_INVALID_ARG
    assert call(K=128, y=None) == salr.SALR_ERR_INVALID_ARG
    assert call(K=128, R=300) == salr.SALR_ERR_UNSUPPORTED
    assert call(K=128, nnz=4 * 128 * 8) == salr.SALR_ERR_SHAPE
    assert call(K=128, ws=None) == salr.SALR_ERR_CAPACITY
    assert call(K=128, ws_bytes=256) == salr.SALR_ERR_CAPACITY
    # the entry point without a workspace: same validation, and a size limit of its own
    na = lib.salr_sparse_lowrank_linear_noalloc
    assert na(fake, -1, 64, 8, fake, fake, fake, fake, fake, 4, fake, None) == salr.SALR_ERR_INVALID_ARG
    assert na(fake, 4, 40, 8, fake, fake, fake, fake, fake, 4, fake, None) == salr.SALR_ERR_SHAPE
    assert na(fake, 4, 64, 8, fake, fake, fake, fake, fake, 300, fake, None) == salr.SALR_ERR_UNSUPPORTED
    assert na(fake, 4096, 28672, 8192, fake, fake, fake, fake, fake, 64, fake, None) == salr.SALR_ERR_CAPACITY
    assert na(fake, 0, 64, 8, fake, fake, fake, fake, fake, 4, fake, None) == salr.SALR_OK


def test_slice_table_validation(lib):
    import ctypes
    import paper_2601_16991_amd as salr
    fake = 0x1000   # never dereferenced: every call below fails validation first (or has nothing to do)
    q = lib.salr_slice_table_bytes
    q.restype = ctypes.c_size_t
    assert q(4096, 4096) == 4096 * 8 * 2 * 4
    assert q(0, 4096) == 0 and q(16, 40) == 0 and q(-1, 64) == 0
    b = lib.salr_build_slice_table
    assert b(fake, fake, -1, 64, fake, 1 << 20, None) == salr.SALR_ERR_INVALID_ARG
    assert b(None, fake, 4, 64, fake, 1 << 20, None) == salr.SALR_ERR_INVALID_ARG
    assert b(fake, None, 4, 64, fake, 1 << 20, None) == salr.SALR_ERR_INVALID_ARG
    assert b(fake, fake, 4, 64, None, 1 << 20, None) == salr.SALR_ERR_INVALID_ARG
    assert b(fake, fake, 4, 40, fake, 1 << 20, None) == salr.SALR_ERR_SHAPE
    assert b(fake, fake, 4, 64, fake, 4 * 64 - 1, None) == salr.SALR_ERR_CAPACITY
    assert b(None, None, 0, 64, None, 0, None) == salr.SALR_OK
    p = lib.salr_sparse_lowrank_linear_prepared
    # the table is an input of the prepared call: NULL is refused; otherwise the validation of the plain call
    assert p(fake, 4, 64, 8, fake, fake, fake, None, fake, fake, 4, fake, fake, 1 << 20, None) == salr.SALR_ERR_INVALID_ARG
    assert p(fake, 4, 40, 8, fake, fake, fake, fake, fake, fake, 4, fake, fake, 1 << 20, None) == salr.SALR_ERR_SHAPE
    assert p(fake, 4, 64, 8, fake, fake, fake, fake, fake, fake, 300, fake, fake, 1 << 20, None) == salr.SALR_ERR_UNSUPPORTED
    assert p(fake, 4, 64, 8, fake, fake, fake, fake, fake, fake, 4, fake, None, 0, None) == salr.SALR_ERR_CAPACITY
    assert p(fake, 0, 64, 8, fake, fake, fake, None, fake, fake, 4, fake, None, 0, None) == salr.SALR_OK
