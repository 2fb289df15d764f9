"""Pins for the oracle's bitmap encode / decode (paper Sec. 3.3).  CPU only."""
import numpy as np
import pytest

import oracle
import salr_workloads as wl


def _random_sparse(rows, cols, density, seed):
    rng = np.random.default_rng(seed)
    w = wl.gaussian_bf16((rows, cols), 0.02, seed + 1)
    w[(w & 0x7FFF) == 0] = 0x3F80  # no accidental zeros among candidates
    drop = rng.random((rows, cols)) >= density
    w[drop] = 0
    return w


def _python_encode(w):
    """Element loops straight from the definition: B_nk = [w_nk != 0], v = nonzeros in row-major order."""
    rows, cols = w.shape
    wpr = (cols + 31) // 32
    bitmap = [[0] * wpr for _ in range(rows)]
    values, offsets = [], []
    for n in range(rows):
        offsets.append(len(values))
        for k in range(cols):
            if (int(w[n, k]) & 0x7FFF) != 0:
                bitmap[n][k // 32] |= 1 << (k % 32)
                values.append(int(w[n, k]))
    offsets.append(len(values))
    return bitmap, values, offsets


@pytest.mark.parametrize("rows,cols,density", [(1, 1, 1.0), (1, 1, 0.0), (3, 5, 0.5), (4, 32, 0.5), (5, 33, 0.3),
                                               (7, 100, 0.7), (2, 64, 1.0), (2, 64, 0.0), (9, 31, 0.5)])
def test_encode_matches_element_loops(rows, cols, density):
    w = _random_sparse(rows, cols, density, 100 + rows * cols)
    bitmap, values, offsets = oracle.encode(w)
    pb, pv, po = _python_encode(w)
    assert bitmap.tolist() == pb
    assert values.tolist() == pv
    assert offsets.tolist() == po


def test_round_trip_and_popcounts_tiny_config():
    cfg = wl.CONFIGS["tiny"]
    w = wl.dense_weight(cfg)
    for permille in (500, 700):
        keep = cfg.keep(permille)
        w_hat = oracle.mask_topk_rows(w, keep)
        bitmap, values, offsets = oracle.encode(w_hat)
        pop = np.array([[bin(int(x)).count("1") for x in row] for row in bitmap])
        assert pop.sum() == offsets[-1] == values.size == cfg.N * keep
        assert (np.diff(offsets.astype(np.int64)) == pop.sum(axis=1)).all()
        assert (pop.sum(axis=1) == keep).all()
        assert offsets[0] == 0
        assert (oracle.decode(bitmap, values, offsets, cfg.N, cfg.K) == w_hat).all()
        assert (oracle.decode(bitmap, values, offsets, cfg.N, cfg.K, use_lut=True) == w_hat).all()


def test_round_trip_ragged_columns_and_empty_rows():
    for rows, cols in [(6, 37), (3, 1), (4, 95), (2, 7)]:
        w = _random_sparse(rows, cols, 0.4, rows + cols)
        w[0, :] = 0  # an all-zero row
        bitmap, values, offsets = oracle.encode(w)
        assert offsets[0] == offsets[1] == 0
        # pad bits of the last word are zero
        if cols % 32:
            assert ((bitmap[:, -1] >> np.uint32(cols % 32)) == 0).all()
        for use_lut in (False, True):
            assert (oracle.decode(bitmap, values, offsets, rows, cols, use_lut=use_lut) == w).all()


def test_empty_matrix():
    w = np.zeros((0, 64), dtype=np.uint16)
    bitmap, values, offsets = oracle.encode(w)
    assert bitmap.shape == (0, 2) and values.size == 0 and offsets.tolist() == [0]
    assert oracle.decode(bitmap, values, offsets, 0, 64).shape == (0, 64)


def test_negative_zero_nan_inf():
    # -0.0 is a zero (bit clear, decodes to +0.0); NaN and Inf are nonzero and copied bit for bit
    w = np.array([[0x8000, 0x7FC0, 0x0000, 0xFF80, 0x0001, 0x8001]], dtype=np.uint16)
    bitmap, values, offsets = oracle.encode(w)
    assert bitmap.tolist() == [[0b111010]]
    assert values.tolist() == [0x7FC0, 0xFF80, 0x0001, 0x8001]
    back = oracle.decode(bitmap, values, offsets, 1, 6)
    assert back.tolist() == [[0x0000, 0x7FC0, 0x0000, 0xFF80, 0x0001, 0x8001]]


def test_lut_hand_worked_mask():
    # mask 0b10110010: bits 1, 4, 5, 7 set -> they are the 0th, 1st, 2nd, 3rd nonzero of the block
    lut = oracle.build_lut()
    assert lut[0b10110010].tolist() == [-1, 0, -1, -1, 1, 2, -1, 3]
    assert lut[0].tolist() == [-1] * 8
    assert lut[255].tolist() == list(range(8))
    assert lut[0b00000001].tolist() == [0] + [-1] * 7
    assert lut[0b10000000].tolist() == [-1] * 7 + [0]


def test_lut_equals_prefix_popcount_for_all_masks():
    lut = oracle.build_lut()
    for m in range(256):
        for t in range(8):
            expect = bin(m & ((1 << t) - 1)).count("1") if (m >> t) & 1 else -1
            assert lut[m, t] == expect


def test_byte_view_of_words_is_the_papers_byte_mask():
    # column 8b+t <-> bit t of byte b (little-endian words)
    cols = 64
    for k in (0, 7, 8, 31, 32, 63):
        w = np.zeros((1, cols), dtype=np.uint16)
        w[0, k] = 0x3F80
        bitmap, _, _ = oracle.encode(w)
        as_bytes = bitmap.view(np.uint8).reshape(-1)
        assert as_bytes[k // 8] == 1 << (k % 8)
        assert as_bytes.sum() == 1 << (k % 8)


def test_both_decoders_agree_on_random_data():
    w = _random_sparse(64, 416, 0.5, 5)
    bitmap, values, offsets = oracle.encode(w)
    a = oracle.decode(bitmap, values, offsets, 64, 416)
    b = oracle.decode(bitmap, values, offsets, 64, 416, use_lut=True)
    assert (a == b).all() and (a == w).all()


def test_values_are_row_major_order():
    # distinct values 1..: the compact array must list them in row-major order of their positions
    rows, cols = 5, 40
    rng = np.random.default_rng(3)
    w = np.zeros((rows, cols), dtype=np.uint16)
    pos = np.sort(rng.choice(rows * cols, size=60, replace=False))
    w.reshape(-1)[pos] = np.arange(1, 61, dtype=np.uint16)
    _, values, offsets = oracle.encode(w)
    assert values.tolist() == list(range(1, 61))
    assert offsets.tolist() == [int((pos < n * cols).sum()) for n in range(rows + 1)]
