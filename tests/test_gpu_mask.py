"""GPU parity: salr_magnitude_mask_rows / salr_magnitude_mask_nm through the C boundary vs the CPU
oracle, bit for bit (the masks are integer work on bf16 patterns; ties make the order matter)."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import to_dev_u16, to_host_u16

pytestmark = pytest.mark.gpu


def _salr():
    import paper_2601_16991_amd as salr
    return salr


def _few_magnitudes(shape, seed):
    """Rows drawn from a handful of values, both signs and both zeros: nearly everything ties."""
    rng = np.random.default_rng(seed)
    vals = wl.f32_to_bf16_bits(np.array([0.5, -0.5, 0.25, -0.25, 1.0, -1.0, 0.125, 2.0, 0.0, -0.0], dtype=np.float32))
    return vals[rng.integers(0, len(vals), size=shape)]


def _check_rows(w, keep, label):
    print(f"[mask_rows] {label} shape={w.shape} keep={keep}", flush=True)
    got = _salr().mask_rows(to_dev_u16(w), keep)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(got).reshape(w.shape), oracle.mask_topk_rows(w, keep)), label


@pytest.mark.parametrize("rows,cols,keep", [
    (1, 1, 0), (1, 1, 1), (3, 5, 2), (6, 13, 5), (4, 32, 16), (5, 37, 37), (5, 37, 0), (9, 100, 33),
    (7, 2048, 1024), (3, 2056, 700), (5, 4104, 1231), (2, 6151, 3000), (300, 8, 4), (2, 30720, 15360)])
def test_mask_rows_tie_heavy(rows, cols, keep):
    _check_rows(_few_magnitudes((rows, cols), rows * 1000 + cols), keep, "ties")


@pytest.mark.parametrize("rows,cols,keep", [
    (5, 8, 0), (5, 8, 8), (6, 64, 1), (3, 4096, 4096), (7, 4096, 0), (9, 8192, 4000), (5, 2056, 2055), (1, 520, 13),
    (4, 1024, 512), (6, 3072, 77)])
def test_mask_rows_one_wave_per_row(rows, cols, keep):
    """Rows of up to 8192 columns in whole 8-column units go through the kernel that keeps a row in the registers of
    one wave (four rows per workgroup): row counts that are not multiples of four, the extreme `keep` values, ties."""
    _check_rows(_few_magnitudes((rows, cols), rows * 77 + cols), keep, "wave kernel, ties")
    _check_rows(wl.gaussian_bf16((rows, cols), 0.02, cols + keep + 1), keep, "wave kernel, gaussian")


@pytest.mark.parametrize("rows,cols,keep", [(5, 37, 11), (4, 4096, 2048), (3, 4099, 1230), (2, 14336, 7168)])
def test_mask_rows_gaussian(rows, cols, keep):
    _check_rows(wl.gaussian_bf16((rows, cols), 0.02, cols + keep), keep, "gaussian")


def test_mask_rows_longer_than_the_lds_row_cache():
    # rows beyond 28672 columns are re-read from memory on every pass; vector and ragged widths
    _check_rows(_few_magnitudes((2, 30728), 5), 10000, "global vec")
    _check_rows(wl.gaussian_bf16((2, 40003), 0.02, 6), 20001, "global ragged")


def test_mask_rows_special_values():
    w = wl.gaussian_bf16((4, 256), 0.02, 9)
    w[0, 5] = 0x7FC0   # NaN ranks above everything
    w[0, 9] = 0xFF80   # -Inf
    w[1, :] = 0x8000   # a row of -0.0: whatever is kept stays -0.0, the rest becomes +0.0
    w[2, :] = 0x3F80   # a constant row: the first `keep` columns survive
    _check_rows(w, 100, "special")


def test_mask_rows_config_shapes():
    for name in ("tiny", "llama3_8b_q_proj"):
        cfg = wl.CONFIGS[name]
        w = wl.dense_weight(cfg, rows=min(cfg.N, 96))
        _check_rows(w, cfg.keep(500), name)


def test_mask_rows_then_encode_matches_the_oracle_chain():
    """Mask and encoder chained on the device give the arrays the oracle's chain gives."""
    salr = _salr()
    cfg = wl.CONFIGS["tiny"]
    w = wl.dense_weight(cfg)
    keep = cfg.keep(500)
    rb, rv, ro = oracle.encode(oracle.mask_topk_rows(w, keep))
    bitmap, values, offsets = salr.encode(salr.mask_rows(to_dev_u16(w), keep))
    torch.cuda.synchronize()
    assert np.array_equal(offsets.cpu().numpy().view(np.uint32), ro)
    assert np.array_equal(bitmap.cpu().numpy().view(np.uint32).reshape(rb.shape), rb)
    assert np.array_equal(to_host_u16(values), rv)


@pytest.mark.parametrize("n,m", [(2, 4), (1, 4), (4, 8), (1, 2), (4, 4), (0, 4), (3, 6), (5, 16), (2, 64)])
def test_mask_nm(n, m):
    for rows, groups, gen in [(5, 8, "ties"), (3, 129, "ties"), (7, 64, "gauss"), (1, 1, "ties")]:
        cols = groups * m
        w = _few_magnitudes((rows, cols), n * 100 + m) if gen == "ties" else wl.gaussian_bf16((rows, cols), 0.02, n + m)
        print(f"[mask_nm] {n}:{m} shape={w.shape}", flush=True)
        got = _salr().mask_nm(to_dev_u16(w), n, m)
        torch.cuda.synchronize()
        assert np.array_equal(to_host_u16(got).reshape(w.shape), oracle.mask_nm(w, n, m)), (n, m, rows, cols)


def test_mask_nm_q_proj_2_of_4():
    cfg = wl.CONFIGS["llama3_8b_q_proj"]
    w = wl.dense_weight(cfg, rows=256)
    got = _salr().mask_nm(to_dev_u16(w), 2, 4)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(got).reshape(w.shape), oracle.mask_nm(w, 2, 4))
