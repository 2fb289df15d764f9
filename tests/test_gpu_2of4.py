"""GPU parity: the layer on 2:4-masked weights through salr_sparse_lowrank_linear_2of4 (sparse matrix-core
instructions on bitmap and packed values as they are) vs the fp64 CPU oracle, and the check salr_bitmap_is_2of4.

Bar: max |Y - Y_ref| <= 1e-2 * max |Y_ref|, as for salr_sparse_lowrank_linear."""
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


def _problem(M, K, N, ranks, seed, std_ab=0.05):
    """X, a 2:4-masked weight (Gaussian: no exact zeros among the kept values), concatenated adapters."""
    x = wl.gaussian_bf16((M, K), 1.0, seed + 1)
    w_hat = oracle.mask_nm(wl.gaussian_bf16((N, K), 0.02, seed + 2), 2, 4)
    As = [wl.gaussian_bf16((K, r), std_ab, seed + 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), std_ab, seed + 20 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = wl.concat_adapters(As, Bs) if ranks else (None, None)
    return x, w_hat, a_cat, b_cat


def _run(x, w_hat, a_cat, b_cat):
    salr = _salr()
    rb, rv, ro = oracle.encode(w_hat)
    y = salr.linear_2of4(to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro),
                         None if a_cat is None else to_dev_u16(a_cat), None if b_cat is None else to_dev_u16(b_cat))
    torch.cuda.synchronize()
    return y_to_f64(y)


def _assert_close(y, y_ref, label):
    scale = float(np.max(np.abs(y_ref)))
    err = float(np.max(np.abs(y - y_ref)))
    print(f"[2of4] {label}: max|d|={err:.3e} scale={scale:.3e} rel={err / scale if scale else 0:.2e}", flush=True)
    assert err <= REL_TOL * scale + 1e-30, f"{label}: {err} > {REL_TOL} * {scale}"


@pytest.mark.parametrize("M,K,N,ranks", [
    (1, 128, 16, ()),                 # one chunk, one row tile, a single token
    (16, 512, 132, (8,)),             # the second row tile holds 4 rows
    (33, 1024, 260, (16, 16)),        # K split in 2, 4 m-tiles
    (64, 4096, 96, ()),               # K split in 8, two waves of the tile past N
    (128, 2048, 516, (40, 60)),       # 8 m-tiles, four rank steps
    (100, 384, 1000, (5,)),           # three chunks, ragged M
    (9, 256, 8196, (4,)),             # many row tiles
    (16, 1024, 28676, (8,)),          # 225 row tiles
    (48, 16384, 64, (4,)),            # K split in 16
    (20, 640, 130, (8,)),             # N % 4 != 0 with few row tiles: the general path
    (16, 96, 64, (8,)),               # K % 128 != 0: the general path
    # M > 128 where the tiles fill the chip: the tiled GEMM on the sparse MFMA (k-steps of 64 columns)
    (129, 64, 8196, (3,)),            # 128 x 128 tiles: one k-step; 2 x 65 tiles, the last ones almost empty
    (300, 256, 8400, (16, 16)),       # ragged in both tile dimensions, 3 x 66 tiles, four k-steps
    (1000, 128, 8192, (40, 60)),      # 8 x 64 tiles, four rank steps
    (256, 128, 8192, ()),             # exact tiles, no adapters
    (1000, 64, 3100, (8,)),           # a layer of fewer than 8192 rows with 8 x 25 tiles of 128 x 128
    (3500, 64, 3580, (8,)),           # 256 x 224 tiles (14 x 16 of them: one round of the CUs), ragged in both dimensions
    (3585, 128, 3588, (16, 16)),      # 256 x 224 tiles, one token and four rows in the last ones
    (3900, 64, 3836, (8,)),           # 256 x 256 tiles (16 x 15: one round; 224-wide ones would need two), ragged
    # M > 128 with too few tiles: the general path
    (200, 256, 64, (8,)),
    (1000, 1024, 260, (40, 60)),
    (257, 128, 513, (7,)),            # N % 4 != 0: the general path
    (160, 96, 64, (8,)),              # K % 64 != 0: the general path
    (128, 256, 128, (128, 128)),      # rank 256 with 128 tokens
    (40, 1280, 8320, ()),             # N % 4 == 0 but ragged last tile, no adapters
    (31, 256, 8191, (3,)),            # N % 4 != 0 with many row tiles: scalar stores
])
def test_linear_2of4_shapes(M, K, N, ranks):
    x, w_hat, a_cat, b_cat = _problem(M, K, N, ranks, 7 * M + K + 3 * N)
    _assert_close(_run(x, w_hat, a_cat, b_cat), oracle.linear(x, w_hat, a_cat, b_cat), f"M{M} K{K} N{N} R{sum(ranks)}")


def test_identity_activations_read_out_weights_exactly():
    """X = I: Y rows are columns of What (exactly representable), so the result is bit-exact: every stored value
    lands on the column its two index bits name."""
    K, N = 128, 48
    _, w_hat, _, _ = _problem(1, K, N, (), 11)
    eye = wl.f32_to_bf16_bits(np.eye(K, dtype=np.float32))
    y = _run(eye, w_hat, None, None)
    assert np.array_equal(y, oracle.bf16_to_f64(w_hat).T)


def test_every_pair_of_positions():
    """Rows built from the six ways to place two values in a group of four, each group with its own values."""
    K, N, M = 128, 16, 4
    pairs = [(0, 1), (0, 2), (1, 2), (0, 3), (1, 3), (2, 3)]
    rng = np.random.default_rng(3)
    w = np.zeros((N, K), dtype=np.float32)
    for n in range(N):
        for grp in range(K // 4):
            p = pairs[(n + 5 * grp + grp // 7) % 6]
            w[n, 4 * grp + p[0]] = rng.uniform(0.5, 1.5) * (1 if (n + grp) % 2 else -1)
            w[n, 4 * grp + p[1]] = rng.uniform(0.5, 1.5) * (1 if grp % 3 else -1)
    w_hat = wl.f32_to_bf16_bits(w)
    x = wl.gaussian_bf16((M, K), 1.0, 5)
    _assert_close(_run(x, w_hat, None, None), oracle.linear(x, w_hat, None, None), "all position pairs")


def test_full_size_sampled_rows():
    """Full-size launch (gate/up, 16 and 64 tokens) under the 2:4 mask; the oracle checks a sample of tokens across all N."""
    cfg = wl.CONFIGS["llama3_8b_gate_up_proj"]
    w_hat = oracle.mask_nm(wl.dense_weight(cfg), 2, 4)
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    for M in (16, 64):
        x = wl.activations(cfg, M)
        y = _run(x, w_hat, a_cat, b_cat)
        rows = np.unique(np.minimum(np.array([0, 7, 15, 16, M - 1]), M - 1))
        y_ref = oracle.linear(np.ascontiguousarray(x[rows]), w_hat, a_cat, b_cat)
        _assert_close(y[rows], y_ref, f"gate/up 2:4 M={M} ({len(rows)} sampled tokens)")
        assert np.isfinite(y).all()


def test_prefill_full_size_sampled_rows():
    """Full-size launch of the tiled GEMM (gate/up, 2048 tokens, 2:4 mask); the oracle checks a sample of tokens."""
    cfg = wl.CONFIGS["llama3_8b_gate_up_proj"]
    M = 2048
    w_hat = oracle.mask_nm(wl.dense_weight(cfg), 2, 4)
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    x = wl.activations(cfg, M)
    y = _run(x, w_hat, a_cat, b_cat)
    rows = np.array([0, 1, 63, 64, 127, 128, 777, 2047])
    y_ref = oracle.linear(np.ascontiguousarray(x[rows]), w_hat, a_cat, b_cat)
    _assert_close(y[rows], y_ref, "gate/up 2:4 M=2048 (8 sampled tokens)")
    assert np.isfinite(y).all()


def test_bitmap_check():
    salr = _salr()
    w24 = oracle.mask_nm(wl.gaussian_bf16((64, 256), 0.02, 1), 2, 4)
    rb, _, _ = oracle.encode(w24)
    assert salr.bitmap_is_2of4(to_dev_u32(rb))
    wtop = oracle.mask_topk_rows(wl.gaussian_bf16((64, 256), 0.02, 2), 128)
    rb2, _, _ = oracle.encode(wtop)
    assert not salr.bitmap_is_2of4(to_dev_u32(rb2))
    # one group with a single value, one with three: both fail although the row count is unchanged
    w_bad = w24.copy()
    grp = w_bad[63, 252:256]
    nz = np.flatnonzero(grp)
    grp[nz[0]] = 0
    assert not salr.bitmap_is_2of4(to_dev_u32(oracle.encode(w_bad)[0]))
    w_bad2 = w24.copy()
    z = np.flatnonzero(w_bad2[0, 0:4] == 0)
    w_bad2[0, z[0]] = 0x3C00
    assert not salr.bitmap_is_2of4(to_dev_u32(oracle.encode(w_bad2)[0]))
    # 1:4 and 4:8 masks are not 2:4 either (4:8 keeps four of eight, not two of every four)
    w48 = oracle.mask_nm(wl.gaussian_bf16((32, 256), 0.02, 3), 4, 8)
    assert bool(salr.bitmap_is_2of4(to_dev_u32(oracle.encode(w48)[0]))) == bool(
        all(np.count_nonzero(w48.reshape(-1, 4), axis=1) == 2))


def test_weight_that_fails_the_check_stays_in_bounds():
    """The call does not check its precondition; on a weight that fails it the values are unspecified, but offsets are
    clamped to the stored count: the call completes and writes all of Y."""
    salr = _salr()
    M, K, N = 16, 512, 256
    w = oracle.mask_topk_rows(wl.gaussian_bf16((N, K), 0.02, 9), 100)   # fewer values than 2:4 would store
    rb, rv, ro = oracle.encode(w)
    x = wl.gaussian_bf16((M, K), 1.0, 10)
    y = salr.linear_2of4(to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), None, None)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (M, N)


@pytest.mark.parametrize("M,K,N", [(8, 1024, 2048), (64, 1024, 520)])
def test_graph_replays(M, K, N):
    """A captured call (the barrier-free kernel; the row-tiled one with its reducing pass) is replayed with new
    activations in place; eager work and synchronisations run between replays, and every replay is checked."""
    salr = _salr()
    ranks = (32, 16)
    x0, w_hat, a_cat, b_cat = _problem(M, K, N, ranks, seed=4343)
    rb, rv, ro = oracle.encode(w_hat)
    bm, v, rod = to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro)
    a, b = to_dev_u16(a_cat), to_dev_u16(b_cat)
    x_dev = to_dev_u16(x0)
    y = torch.empty((M, N), dtype=x_dev.dtype, device=dev())
    ws = torch.empty(max(salr.salr_linear_2of4_workspace_bytes(M, K, N, sum(ranks)), 256), dtype=torch.uint8, device=dev())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # one eager call first, as a capture's warm-up
        salr.salr_sparse_lowrank_linear_2of4(x_dev, bm, v, rod, a, b, y, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        salr.salr_sparse_lowrank_linear_2of4(x_dev, bm, v, rod, a, b, y, ws)
    for replay in range(4):
        x = wl.gaussian_bf16((M, K), 0.5 + replay, 8200 + replay)
        x_dev.copy_(to_dev_u16(x))
        graph.replay()
        torch.cuda.synchronize()
        _assert_close(y_to_f64(y), oracle.linear(x, w_hat, a_cat, b_cat), f"graph replay {replay}")
        eager = salr.linear_2of4(x_dev, bm, v, rod, a, b)   # eager work between the replays, on another workspace
        torch.cuda.synchronize()
        assert torch.equal(eager.view(torch.int16), y.view(torch.int16)), f"replay {replay} differs from eager"
