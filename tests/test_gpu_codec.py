"""GPU parity: salr_encode_bitmap / salr_decode through the C boundary vs the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import dev, to_dev_u16, to_dev_u32, to_host_u16, to_host_u32

pytestmark = pytest.mark.gpu


def _salr():
    import paper_2601_16991_amd as salr
    return salr


def _random_sparse(rows, cols, density, seed):
    rng = np.random.default_rng(seed)
    w = wl.gaussian_bf16((rows, cols), 0.02, seed + 1)
    w[(w & 0x7FFF) == 0] = 0x3F80
    w[rng.random((rows, cols)) >= density] = 0
    return w


def _check_codec(w_hat, label):
    salr = _salr()
    print(f"[codec] {label} shape={w_hat.shape}", flush=True)
    rows, cols = w_hat.shape
    rb, rv, ro = oracle.encode(w_hat)
    bitmap, values, offsets = salr.encode(to_dev_u16(w_hat))
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u32(offsets), ro), f"{label}: row_offsets"
    assert np.array_equal(to_host_u32(bitmap).reshape(rb.shape), rb), f"{label}: bitmap"
    assert np.array_equal(to_host_u16(values), rv), f"{label}: values"
    # decode from the ORACLE's arrays (independent of the GPU encoder) and from the GPU's own
    out = salr.decode(to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), rows, cols)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(out).reshape(w_hat.shape), oracle.decode(rb, rv, ro, rows, cols)), f"{label}: decode"
    out2 = salr.decode(bitmap, values, offsets, rows, cols)
    torch.cuda.synchronize()
    expect = w_hat.copy()
    expect[(expect & 0x7FFF) == 0] = 0
    assert np.array_equal(to_host_u16(out2).reshape(w_hat.shape), expect), f"{label}: round trip"


@pytest.mark.parametrize("rows,cols,density", [
    (1, 1, 1.0), (1, 1, 0.0), (3, 5, 0.5), (5, 37, 0.4), (4, 32, 0.5), (9, 100, 0.7), (2, 64, 1.0), (2, 64, 0.0),
    (7, 2048, 0.5), (3, 2056, 0.5), (5, 4104, 0.3), (2, 6151, 0.5), (64, 416, 0.5), (300, 8, 0.5), (17, 24, 0.9)])
def test_codec_small_and_ragged(rows, cols, density):
    w = _random_sparse(rows, cols, density, 1000 + rows * 31 + cols)
    if rows > 2:
        w[1, :] = 0  # an empty row in the middle
    _check_codec(w, f"ragged {rows}x{cols} d={density}")


def test_codec_special_patterns():
    w = np.array([[0x8000, 0x7FC0, 0x0000, 0xFF80, 0x0001, 0x8001, 0x0000, 0x8000, 0x3F80]], dtype=np.uint16)
    _check_codec(w, "neg-zero / nan / inf / denormal")


def test_codec_dense_groups_off_vector_boundaries():
    """Fully dense 512-column groups whose values start at every offset 0..7 inside a 16-byte vector: the
    decoder stages up to 65 vectors for such a group."""
    w = _random_sparse(9, 1544, 1.0, 4242)          # 3 groups of 512 + a ragged fourth of 8 columns
    for r in range(8):
        w[r, :r] = 0                                  # row r has r zeros: row r + 1 starts at offset (...) % 8 != 0
    _check_codec(w, "dense groups, odd starts")


def test_codec_empty():
    salr = _salr()
    w = torch.zeros((0, 64), dtype=torch.int16, device=dev())
    bitmap, values, offsets = salr.encode(w)
    torch.cuda.synchronize()
    assert to_host_u32(offsets).tolist() == [0] and values.numel() == 0
    w = torch.zeros((5, 0), dtype=torch.int16, device=dev())
    bitmap, values, offsets = salr.encode(w)
    torch.cuda.synchronize()
    assert to_host_u32(offsets).tolist() == [0] * 6


@pytest.mark.parametrize("permille", [500, 700])
def test_codec_tiny_config(permille):
    cfg = wl.CONFIGS["tiny"]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(permille))
    _check_codec(w_hat, f"tiny p={permille}")


def test_encode_capacity_never_overrun():
    salr = _salr()
    w = _random_sparse(16, 256, 0.5, 77)
    rb, rv, ro = oracle.encode(w)
    cap = rv.size // 2
    guard = 64
    buf = torch.full((cap + guard,), 0x5A5A, dtype=torch.int16, device=dev())
    bitmap = torch.empty((16, 8), dtype=torch.int32, device=dev())
    offsets = torch.empty(17, dtype=torch.int32, device=dev())
    salr.salr_encode_bitmap(to_dev_u16(w), bitmap, buf[:cap], offsets)
    torch.cuda.synchronize()
    got = to_host_u16(buf)
    assert np.array_equal(got[:cap], rv[:cap])
    assert (got[cap:] == 0x5A5A).all()
    assert np.array_equal(to_host_u32(offsets), ro)  # true counts are still reported


@pytest.mark.parametrize("name,permille,rows", [
    ("llama3_8b_q_proj", 500, None),
    ("llama3_8b_down_proj", 700, 512),     # keep = 4301 per row: odd, unaligned row starts
    ("llama3_8b_down_proj", 500, 256),
    ("llama3_70b_down_proj", 500, 128),    # K = 28672
])
def test_codec_config_shapes(name, permille, rows):
    cfg = wl.CONFIGS[name]
    w = wl.dense_weight(cfg, rows=rows)
    w_hat = oracle.mask_topk_rows(w, cfg.keep(permille))
    _check_codec(w_hat, f"{name} p={permille} rows={w.shape[0]}")
