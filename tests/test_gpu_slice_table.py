"""GPU parity for the prepared-layer path through the C boundary: the slice table (a derived index of the format of
Sec. 3.3: where the packed values of a column range start) bit for bit against the oracle, and the layer called with the
table against the fp64 oracle (max |Y - Y_ref| <= 1e-2 * max |Y_ref|) and bit for bit against the call without it."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import dev, to_dev_u16, to_dev_u32, y_to_f64

pytestmark = pytest.mark.gpu
REL_TOL = 1e-2


def _salr():
    import paper_2601_16991_amd as salr
    return salr


def _weight(N, K, density, seed):
    rng = np.random.default_rng(seed)
    w = wl.gaussian_bf16((N, K), 0.02, seed + 2)
    w[rng.random((N, K)) >= density] = 0
    return w


@pytest.mark.parametrize("N,K,density", [(1, 32, 0.5), (5, 128, 0.5), (37, 1056, 0.3), (100, 4096, 0.5), (33, 4000 + 32, 0.7),
                                         (64, 8192, 0.5), (7, 14336, 0.3), (3, 28672, 1.0), (50, 96, 0.05)])
def test_slice_table_bit_exact(N, K, density):
    salr = _salr()
    w = _weight(N, K, density, 300 + N + K)
    if N > 2:
        w[1, :] = 0   # an empty row
    rb, rv, ro = oracle.encode(w)
    table = salr.build_slice_table(to_dev_u32(rb), to_dev_u32(ro), K)
    torch.cuda.synchronize()
    got = table.cpu().numpy().view(np.uint32)
    assert np.array_equal(got, oracle.slice_table(rb, ro, K)), f"N={N} K={K}"


# shapes that reach every table-fed instantiation of the small-batch kernel (one, two and four row tiles of tokens;
# two and four chunks in flight), shapes whose path has no use for the table (ragged rows, the row-tiled, long-row and
# large-batch kernels), a ragged last row group, no adapters, dense and nearly empty weights
@pytest.mark.parametrize("M,K,N,ranks,density", [
    (1, 128, 16, (8,), 0.5), (16, 1024, 520, (32,), 0.5), (5, 4096, 100, (16, 16), 0.5), (16, 4096, 4096, (32,), 0.5),
    (3, 2048, 8200, (8,), 0.5), (8, 1024, 9000, (), 0.5), (24, 1024, 333, (5,), 0.5), (32, 4096, 1000, (32, 32), 0.3),
    (40, 512, 1001, (16,), 0.5), (64, 2048, 131, (64,), 0.5), (16, 8192, 96, (64,), 0.5), (4, 1024, 64, (4,), 1.0),
    (16, 1024, 64, (4,), 0.05), (7, 1056, 48, (8,), 0.5), (64, 1024, 1024, (32,), 0.5), (8, 14336, 64, (64,), 0.5),
    (130, 256, 70, (8,), 0.5),
    # long rows (the kernel for K >= 12288): one, four and eight groups of chunks per wave, dense and nearly empty rows
    (1, 28672, 40, (64,), 0.5), (16, 12288, 48, (8,), 0.5), (3, 16384, 33, (), 1.0), (8, 32768, 20, (16,), 0.05),
    (16, 14336, 130, (32, 32), 0.7),
    # the row-tiled kernel takes its cursors from the table when K is split 1, 2, 4 or 8 ways (and not when 16 ways)
    (16, 2048, 8200, (8,), 0.5), (128, 4096, 520, (32,), 0.5), (40, 14336, 256, (16,), 0.5), (100, 1024, 2048, (4,), 0.3),
    (33, 8192, 1024, (64,), 0.5),
    # more row groups than CUs on rows of 4096 / 8192 columns, up to 16 tokens, ragged last group; without adapters the
    # plain call has no table, so the bit comparison below is between the table-fed and the plain variant of the kernel
    (1, 4096, 4117, (32,), 0.5), (16, 4096, 4200, (), 0.5), (7, 8192, 4128, (64,), 0.5), (16, 8192, 4113, (), 0.3),
    (3, 4096, 8200, (8,), 0.9), (5, 4096, 12000, (), 1.0), (16, 4096, 6000, (16, 16), 0.5)])
def test_prepared_linear(M, K, N, ranks, density):
    salr = _salr()
    seed = 9000 + M + K + N
    x = wl.gaussian_bf16((M, K), 1.0, seed + 1)
    w = _weight(N, K, density, seed)
    As = [wl.gaussian_bf16((K, r), 0.01, seed + 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), 0.01, seed + 20 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = wl.concat_adapters(As, Bs) if ranks else (None, None)
    rb, rv, ro = oracle.encode(w)
    bm, v, rod = to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro)
    a = None if a_cat is None else to_dev_u16(a_cat)
    b = None if b_cat is None else to_dev_u16(b_cat)
    table = salr.build_slice_table(bm, rod, K)
    print(f"[prepared] M{M} K{K} N{N} R{sum(ranks)} density {density}", flush=True)
    y_t = salr.linear_prepared(to_dev_u16(x), bm, v, rod, table, a, b)
    y_0 = salr.linear(to_dev_u16(x), bm, v, rod, a, b)
    torch.cuda.synchronize()
    y_ref = oracle.linear(x, w, a_cat, b_cat)
    scale = float(np.max(np.abs(y_ref)))
    err = float(np.max(np.abs(y_to_f64(y_t) - y_ref)))
    print(f"[prepared] max|d|={err:.3e} scale={scale:.3e}", flush=True)
    assert err <= REL_TOL * scale + 1e-30
    assert torch.equal(y_t.view(torch.int16), y_0.view(torch.int16)), "the table changes where values are found, not the sums"


def test_prepared_full_size_q_proj_sampled_against_unprepared():
    """The headline layer at full size in the launch configuration the bench times: with and without the table, all
    outputs bit for bit; the call without it is checked against the oracle in tests/test_gpu_linear_configs.py."""
    salr = _salr()
    cfg = wl.CONFIGS["llama3_8b_q_proj"]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    rb, rv, ro = oracle.encode(w_hat)
    bm, v, rod = to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro)
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    a, b = to_dev_u16(a_cat), to_dev_u16(b_cat)
    table = salr.build_slice_table(bm, rod, cfg.K)
    torch.cuda.synchronize()
    assert np.array_equal(table.cpu().numpy().view(np.uint32), oracle.slice_table(rb, ro, cfg.K))
    for M in (1, 4, 16, 64):
        x = to_dev_u16(wl.activations(cfg, M))
        y_t = salr.linear_prepared(x, bm, v, rod, table, a, b)
        y_0 = salr.linear(x, bm, v, rod, a, b)
        torch.cuda.synchronize()
        assert torch.equal(y_t.view(torch.int16), y_0.view(torch.int16)), f"M={M}"
