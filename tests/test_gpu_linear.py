"""GPU parity: salr_sparse_lowrank_linear through the C boundary vs the fp64 CPU oracle.

Bar: max |Y - Y_ref| <= 1e-2 * max |Y_ref| (bf16 inputs, fp32 accumulation, bf16 output)."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import dev, to_dev_u16, to_dev_u32, to_host_u16, y_to_f64

pytestmark = pytest.mark.gpu

REL_TOL = 1e-2


def _salr():
    import paper_2601_16991_amd as salr
    return salr


def _run(x, w_hat, a_cat, b_cat):
    salr = _salr()
    rb, rv, ro = oracle.encode(w_hat)
    y = salr.linear(to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro),
                    None if a_cat is None else to_dev_u16(a_cat), None if b_cat is None else to_dev_u16(b_cat))
    torch.cuda.synchronize()
    return y_to_f64(y)


def _assert_close(y, y_ref, label, rel=REL_TOL):
    scale = float(np.max(np.abs(y_ref))) if y_ref.size else 0.0
    err = float(np.max(np.abs(y - y_ref))) if y_ref.size else 0.0
    print(f"[linear] {label}: max|d|={err:.3e} scale={scale:.3e} rel={err / scale if scale else 0:.2e}", flush=True)
    assert err <= rel * scale + 1e-30, f"{label}: {err} > {rel} * {scale}"


def _problem(M, K, N, ranks, seed, density=0.5, std_ab=0.01):
    rng = np.random.default_rng(seed)
    x = wl.gaussian_bf16((M, K), 1.0, seed + 1)
    w = wl.gaussian_bf16((N, K), 0.02, seed + 2)
    w[rng.random((N, K)) >= density] = 0
    As = [wl.gaussian_bf16((K, r), std_ab, seed + 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), std_ab, seed + 20 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = wl.concat_adapters(As, Bs) if ranks else (None, None)
    return x, w, a_cat, b_cat


def test_tiny_config():
    cfg = wl.CONFIGS["tiny"]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    x = wl.activations(cfg, cfg.Ms[0])
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    _assert_close(_run(x, w_hat, a_cat, b_cat), oracle.linear(x, w_hat, a_cat, b_cat), "tiny")


@pytest.mark.parametrize("M,K,N,ranks", [
    (1, 64, 16, (8,)), (3, 96, 40, (4, 4)), (17, 128, 100, (16, 16)), (65, 256, 130, (5,)), (100, 32, 64, (33,)),
    (16, 512, 64, ()), (130, 160, 70, (64, 64, 64, 64)), (2, 2048, 48, (1,)), (64, 64, 64, (32,)),
    # M > 64 with K % 64 == 0: decode once into dense scratch, then the dense MFMA kernel (1, 2, 3, 5 k-steps;
    # ragged in both tile dimensions); other K at such M fall back to the generic kernel
    (200, 512, 300, (16, 16)), (255, 128, 513, (7,)), (70, 384, 64, ()), (65, 1024, 1030, (40, 60)),
    (129, 64, 129, (3,)), (160, 192, 260, (16,)),
    (300, 512, 300, (16, 16)), (257, 128, 513, (7,)), (600, 192, 260, (16,)), (256, 64, 129, (3,)),
    (1030, 64, 100, ()), (1100, 128, 257, (16, 16)), (1025, 192, 140, (33,)), (1024, 320, 130, (5,)),
    (1024, 32, 130, (5,)), (1100, 96, 70, (16,)),
    # few output tiles and a long K: the dense stage splits K over 2, 4 or 8 workgroups per tile (fp32 partials)
    (300, 1024, 260, (16,)), (256, 2048, 128, (8, 8)), (512, 512, 100, ()), (257, 4096, 36, (3,)),
    # M in 17..64: the streaming path with 2 and 4 m-tiles
    (33, 640, 50, (8,)), (48, 4096, 32, (16, 16)), (64, 96, 17, ()),
    # more than 512 row groups: the streaming variant that shares a CU between two workgroups
    (3, 256, 8200, (8,)), (16, 1024, 8192, (16, 16)),
])
def test_ragged_shapes(M, K, N, ranks):
    x, w, a_cat, b_cat = _problem(M, K, N, ranks, 31 * M + K + N, std_ab=0.05)
    _assert_close(_run(x, w, a_cat, b_cat), oracle.linear(x, w, a_cat, b_cat), f"M{M} K{K} N{N} R{sum(ranks)}")


@pytest.mark.parametrize("M,K,N,ranks,density", [
    # 17..128 tokens on whole 128-column chunks: the row-tiled streaming path (128 weight rows per workgroup, X tile in LDS)
    (33, 128, 132, (8,), 0.5),            # one chunk; the second row tile holds 4 rows
    (64, 1024, 260, (16, 16), 0.5),       # K split in 2: fp32 partials, adapters ride with slice 0
    (128, 2048, 516, (40, 60), 0.5),      # 8 m-tiles, K split in 4, four rank steps
    (100, 384, 1000, (5,), 0.5),          # three chunks, ragged M
    (40, 4096, 96, (), 0.5),              # K split in 8, two waves of the tile past N, no adapters
    (17, 512, 8320, (8, 8), 0.5),         # 9..32 tokens take this path on layers of 8192 rows and more
    (9, 256, 8192, (4,), 0.5),
    # many row tiles
    (16, 1024, 28676, (8,), 0.5),         # 225 tiles, the last one with 4 rows; K split in 2 (4 chunks each)
    (40, 2304, 28672, (16, 16), 0.5),     # 224 tiles, 18 chunks split in 2
    (24, 1024, 30000, (), 0.7),           # 2 m-tiles, no adapters
    (48, 16384, 64, (4,), 0.5),           # K split in 16: cursors from popcounts of up to 120 chunks to the left
    (48, 512, 256, (8,), 1.0),            # every bit set: pieces of 128 values (17 vectors, fetched in two goes)
    (80, 1280, 384, (16,), 0.8),          # most chunks longer than the 12 prefetched vectors
    (64, 256, 128, (128, 128), 0.5),      # rank 256 with 64 tokens
    (128, 256, 128, (128, 128), 0.5),     # rank 256 with 128 tokens: T fills the LDS of both X tiles
    (128, 128, 128, (1,), 0.1),           # sparse rows, empty pieces
])
def test_row_tiled_path(M, K, N, ranks, density):
    x, w, a_cat, b_cat = _problem(M, K, N, ranks, 17 * M + K + 3 * N, density=density, std_ab=0.05)
    _assert_close(_run(x, w, a_cat, b_cat), oracle.linear(x, w, a_cat, b_cat), f"row-tiled M{M} K{K} N{N} R{sum(ranks)}")


def test_row_tiled_random_shapes():
    """Seeded random shapes around the row-tiled path's limits (token counts 9..128, 1..20 chunks, ragged row tiles,
    ranks 0..70, sparse to full rows); shapes that fall outside it take the other paths, which must agree as well."""
    rng = np.random.default_rng(2601)
    for case in range(28):
        M = int(rng.integers(9, 129))
        K = 128 * int(rng.integers(1, 21))
        N = int(rng.integers(1, 176)) * 4 if case % 4 else int(rng.integers(4, 700))
        if case % 7 == 0:
            N, K = 8192 + 4 * int(rng.integers(0, 40)), 128 * int(rng.integers(1, 5))
        n_ad = int(rng.integers(0, 4))
        ranks = tuple(int(rng.integers(1, 25)) for _ in range(n_ad))
        density = float(rng.choice([0.1, 0.3, 0.5, 0.75, 0.9, 1.0]))
        x, w, a_cat, b_cat = _problem(M, K, N, ranks, 5000 + case, density=density, std_ab=0.05)
        _assert_close(_run(x, w, a_cat, b_cat), oracle.linear(x, w, a_cat, b_cat),
                      f"random {case}: M{M} K{K} N{N} R{sum(ranks)} density {density}")


@pytest.mark.parametrize("M,K,N,ranks,density", [
    # rows longer than 32 chunks (K > 4096, K % 128 == 0): the small-batch kernel whose waves exchange the nonzero
    # counts of their slices through LDS before the stream starts (16-byte bitmap loads)
    (1, 4224, 48, (8, 8), 0.5),           # 33 chunks over 8 waves: slices of 4 and 5 chunks
    (8, 8192, 100, (32, 32), 0.5),        # 8 chunks per wave, last row group ragged
    (16, 14336, 64, (64,), 0.3),          # K of the down_proj layer: 14 chunks per wave
    (4, 16384, 600, (), 0.5),             # no adapters
    (16, 5120, 48, (16,), 1.0),           # every bit set: pieces of 17 vectors, the two-chunks-in-flight loop
    (3, 28672, 48, (64,), 0.5),           # K of the 70B down_proj layer: 28 chunks per wave
    (2, 4352, 16, (1,), 0.05),            # sparse rows: many empty pieces
    # from K = 12288 on: the kernel that loads every bitmap word once and takes a row's values four chunks at a time
    (8, 12288, 40, (8,), 1.0),            # every bit set: pieces of 65 vectors, 25 of them fetched when consumed
    (2, 16384, 32, (1,), 0.05),           # sparse rows: empty pieces
    (16, 12416, 20, (16, 16), 0.75),      # 97 chunks over 8 waves: slices of 12 and 13 chunks, last group ragged
    (9, 32768, 18, (), 0.5),              # the longest rows the kernel takes: 8 groups per wave
    (5, 32896, 18, (4,), 0.5),            # one chunk more: back to the small-batch kernel
    # ... with >= 512 row groups: two workgroups per CU, two chunks in flight
    (1, 4224, 8200, (8, 8), 0.5),
    (8, 8192, 8192, (64,), 0.5),
    (5, 4480, 8300, (), 0.3),
    (8, 4608, 8192, (16, 16), 1.0),
    # ... with 17 to 32 tokens (two row tiles of X, three chunks in flight)
    (24, 8192, 100, (32, 32), 0.5),
    (32, 4224, 48, (), 0.7),
    (17, 6144, 200, (8,), 1.0),
    # bitmap rows that are no multiple of 16 bytes (K % 128 != 0) and many chunks: scalar bitmap loads, same exchange
    (4, 4032, 40, (8,), 0.5), (16, 8224, 33, (32,), 0.5), (40, 4128, 50, (4,), 0.5), (64, 4192, 20, (), 1.0),
])
def test_small_batch_long_rows(M, K, N, ranks, density):
    x, w, a_cat, b_cat = _problem(M, K, N, ranks, 13 * M + K + 7 * N, density=density, std_ab=0.05)
    _assert_close(_run(x, w, a_cat, b_cat), oracle.linear(x, w, a_cat, b_cat),
                  f"long rows M{M} K{K} N{N} R{sum(ranks)} density {density}")


def _run_lean(x, w_hat, a_cat, b_cat):
    """The call with the least workspace it accepts: large batches then keep no decoded copy of the weight."""
    salr = _salr()
    M, K = x.shape
    N = w_hat.shape[0]
    R = 0 if a_cat is None else a_cat.shape[1]
    rb, rv, ro = oracle.encode(w_hat)
    least = salr.salr_linear_workspace_bytes_min(M, K, N, R)
    assert least < salr.salr_linear_workspace_bytes(M, K, N, R)
    ws = torch.randint(0, 256, (max(least, 256),), dtype=torch.uint8, device=dev())[:least]
    y = salr.linear(to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro),
                    None if a_cat is None else to_dev_u16(a_cat), None if b_cat is None else to_dev_u16(b_cat),
                    workspace=ws if least else torch.empty(0, dtype=torch.uint8, device=dev()))
    torch.cuda.synchronize()
    return y_to_f64(y)


@pytest.mark.parametrize("M,K,N,ranks,density", [
    # M > 64 with K % 64 == 0 and a workspace without room for the decoded weight: decode stage and MFMA stage in one
    # kernel (256 x 128 tiles, double-buffered LDS); ragged in both tile dimensions, 1 to 64 chunks of 64 columns
    (200, 512, 300, (16, 16), 0.5), (255, 128, 513, (7,), 0.5), (70, 320, 64, (), 0.5), (65, 960, 1030, (40, 60), 0.5),
    (1030, 64, 100, (), 0.5), (300, 1024, 260, (16,), 0.5), (600, 192, 260, (16,), 0.5), (129, 64, 129, (3,), 0.5),
    (257, 4096, 36, (3,), 0.5), (512, 512, 100, (), 1.0), (300, 640, 140, (8,), 0.95), (260, 256, 130, (4, 4), 0.05),
    (256, 2048, 128, (128, 128), 0.3),
])
def test_large_batch_without_decoded_copy(M, K, N, ranks, density):
    x, w, a_cat, b_cat = _problem(M, K, N, ranks, 11 * M + K + 5 * N, density=density, std_ab=0.05)
    _assert_close(_run_lean(x, w, a_cat, b_cat), oracle.linear(x, w, a_cat, b_cat),
                  f"fused M{M} K{K} N{N} R{sum(ranks)} density {density}")


def test_gate_up_prefill_without_decoded_copy_sampled_rows():
    """Full-size launch of the fused kernel (M = 2048 on the gate/up layer); the oracle checks 8 rows of X across all N."""
    cfg = wl.CONFIGS["llama3_8b_gate_up_proj"]
    M = cfg.Ms[0]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    x = wl.activations(cfg, M)
    y = _run_lean(x, w_hat, a_cat, b_cat)
    rows = np.array([0, 1, 255, 256, 777, 1024, 2046, 2047])
    _assert_close(y[rows], oracle.linear(np.ascontiguousarray(x[rows]), w_hat, a_cat, b_cat), "gate/up M=2048 fused (8 sampled rows)")
    assert np.isfinite(y).all()


@pytest.mark.parametrize("M,N", [(4096, 3584), (4090, 3580)])
def test_many_tiles_224_wide(M, N):
    """16 row blocks x 14 column blocks of 256 x 256 would leave the second round of the 256 CUs mostly empty;
    the dense stage then takes 256 x 224 tiles (16 x 16 of them).  Short K keeps the oracle cheap."""
    x, w, a_cat, b_cat = _problem(M, 128, N, (8, 8), 5 * M + N, std_ab=0.05)
    _assert_close(_run(x, w, a_cat, b_cat), oracle.linear(x, w, a_cat, b_cat), f"M{M} N{N} 224-wide tiles")


def test_adapter_term_alone():
    """What = 0 isolates (X A_cat) B_cat: the tolerance is then relative to the adapter term itself."""
    x, w, a_cat, b_cat = _problem(16, 512, 256, (16, 16), 5)
    z = np.zeros_like(w)
    _assert_close(_run(x, z, a_cat, b_cat), oracle.linear(x, z, a_cat, b_cat), "adapters only")


def test_adapter_term_by_difference():
    """Y - Y|R=0 against the oracle's adapter term: a mangled adapter cannot hide behind the base product."""
    cfg = wl.CONFIGS["tiny"]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    x = wl.activations(cfg, 16)
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg, std=0.05))
    y_full = _run(x, w_hat, a_cat, b_cat)
    y_base = _run(x, w_hat, None, None)
    ref_delta = oracle.linear(x, np.zeros_like(w_hat), a_cat, b_cat)
    ref_full = oracle.linear(x, w_hat, a_cat, b_cat)
    # two bf16 roundings of Y (each <= 2^-9 relative to |Y|) bound the difference's error
    tol = 2 * 2.0 ** -8 * float(np.max(np.abs(ref_full))) + 1e-2 * float(np.max(np.abs(ref_delta)))
    err = float(np.max(np.abs((y_full - y_base) - ref_delta)))
    print(f"[linear] adapter by difference: err={err:.3e} tol={tol:.3e} |delta|={np.max(np.abs(ref_delta)):.3e}", flush=True)
    assert err <= tol
    assert float(np.max(np.abs(ref_delta))) > 4 * tol  # the check has teeth


@pytest.mark.parametrize("M", [8, 200])
def test_no_adapters_dense_and_empty_weight(M):
    x, w, _, _ = _problem(M, 256, 96, (), 9, density=1.0)   # p = 0: every bit set
    _assert_close(_run(x, w, None, None), oracle.linear(x, w, None, None), "dense bitmap")
    z = np.zeros_like(w)
    y = _run(x, z, None, None)
    assert (y == 0).all()


@pytest.mark.parametrize("M,N,R", [(1, 16, 0), (16, 100, 8), (200, 300, 32)])
def test_empty_contraction_gives_zeros(M, N, R):
    """K == 0: both products are empty sums, so Y = 0 whatever the other operands (which may be null) hold."""
    salr = _salr()
    y = torch.full((M, N), 0x3F80, dtype=torch.int16, device=dev())
    x = torch.empty((M, 0), dtype=torch.int16, device=dev())
    bitmap = torch.empty((N, 0), dtype=torch.int32, device=dev())
    values = torch.empty((0,), dtype=torch.int16, device=dev())
    offsets = torch.zeros(N + 1, dtype=torch.int32, device=dev())
    a_cat = torch.empty((0, R), dtype=torch.int16, device=dev()) if R else None
    b_cat = to_dev_u16(wl.gaussian_bf16((R, N), 1.0, 3)) if R else None
    salr.salr_sparse_lowrank_linear(x, bitmap, values, offsets, a_cat, b_cat, y, None)
    torch.cuda.synchronize()
    assert (to_host_u16(y) == 0).all()


@pytest.mark.parametrize("M", [4, 96])
def test_mixed_density_rows(M):
    """Rows that are empty, dense and in between inside one tile (piece lengths 0 .. 64 per chunk)."""
    x, w, a_cat, b_cat = _problem(M, 512, 80, (8,), 21, density=0.5)
    w[3, :] = 0
    w[5, :] = wl.gaussian_bf16((512,), 0.02, 5)
    w[5, (w[5] & 0x7FFF) == 0] = 0x3C00
    w[7, 100:400] = 0
    w[9, :128] = 0x3C00
    _assert_close(_run(x, w, a_cat, b_cat), oracle.linear(x, w, a_cat, b_cat), f"mixed density M={M}")


def test_identity_activations_read_out_weights_exactly():
    """X = I: Y rows are columns of What (exactly representable), so the result is bit-exact."""
    K, N = 64, 48
    _, w, _, _ = _problem(1, K, N, (), 11)
    eye = wl.f32_to_bf16_bits(np.eye(K, dtype=np.float32))
    y = _run(eye, w, None, None)
    assert np.array_equal(y, oracle.bf16_to_f64(w).T)


def test_q_proj_full_size_all_M():
    cfg = wl.CONFIGS["llama3_8b_q_proj"]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    salr = _salr()
    rb, rv, ro = oracle.encode(w_hat)
    d = (to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), to_dev_u16(a_cat), to_dev_u16(b_cat))
    for M in cfg.Ms:
        x = wl.activations(cfg, M)
        y = salr.linear(to_dev_u16(x), *d)
        torch.cuda.synchronize()
        _assert_close(y_to_f64(y), oracle.linear(x, w_hat, a_cat, b_cat), f"q_proj M={M}")


def test_gate_up_prefill_sampled_rows():
    """Full-size launch (M = 2048); the oracle checks a fixed sample of 8 rows of X across all N."""
    cfg = wl.CONFIGS["llama3_8b_gate_up_proj"]
    M = cfg.Ms[0]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    x = wl.activations(cfg, M)
    y = _run(x, w_hat, a_cat, b_cat)
    rows = np.array([0, 1, 63, 64, 777, 1024, 2046, 2047])
    y_ref = oracle.linear(np.ascontiguousarray(x[rows]), w_hat, a_cat, b_cat)
    _assert_close(y[rows], y_ref, "gate/up M=2048 (8 sampled rows)")
    assert np.isfinite(y).all()


@pytest.mark.parametrize("name,permille,M", [
    ("llama3_8b_down_proj", 700, 512),     # split-K dense stage, odd keep (4301 per row), R = 64
    ("llama3_8b_down_proj", 500, 4096),    # 256 x 256 tiles, T with four row blocks per adapter operand
    ("llama3_70b_attn", 500, 4096),        # K = N = 8192
])
def test_large_batch_full_size_sampled_rows(name, permille, M):
    """Full-size launches of the large-batch path; the oracle checks a fixed sample of 6 rows of X across all N."""
    cfg = wl.CONFIGS[name]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(permille))
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    x = wl.activations(cfg, M)
    y = _run(x, w_hat, a_cat, b_cat)
    rows = np.array([0, 15, 16, 255, M // 2 + 1, M - 1])
    y_ref = oracle.linear(np.ascontiguousarray(x[rows]), w_hat, a_cat, b_cat)
    _assert_close(y[rows], y_ref, f"{name} p={permille} M={M} (6 sampled rows)")
    assert np.isfinite(y).all()


@pytest.mark.parametrize("name,M", [
    ("llama3_8b_gate_up_proj", 16),    # 224 row tiles, K split in 2, one m-tile
    ("llama3_8b_gate_up_proj", 64),    # the same with 4 m-tiles
    ("llama3_8b_down_proj", 128),      # 32 row tiles, K split in 8 (14 chunks each), 8 m-tiles, R = 64
    ("llama3_8b_q_proj", 96),          # 32 row tiles, K split in 8 (4 chunks each)
])
def test_row_tiled_full_size_sampled_rows(name, M):
    """Full-size launches of the row-tiled streaming path; the oracle checks a fixed sample of rows of X across all N."""
    cfg = wl.CONFIGS[name]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    x = wl.activations(cfg, M)
    y = _run(x, w_hat, a_cat, b_cat)
    rows = np.unique(np.minimum(np.array([0, 15, 16, M // 2 + 1, M - 2, M - 1]), M - 1))
    y_ref = oracle.linear(np.ascontiguousarray(x[rows]), w_hat, a_cat, b_cat)
    _assert_close(y[rows], y_ref, f"{name} M={M} ({len(rows)} sampled rows)")
    assert np.isfinite(y).all()


@pytest.mark.parametrize("M,ranks,K", [(1, (8, 8), 512), (16, (32,), 512), (40, (64, 30), 512), (64, (128, 128), 512),
                                       (100, (64, 30), 512), (128, (32,), 2048)])
def test_small_batch_one_workspace_many_calls(M, ranks, K):
    """The small-batch and row-tiled paths keep split-K partial sums of T = X A_cat (and, where K is split over
    workgroups, of Y) in the workspace.  One workspace, first filled with arbitrary bytes, then used by calls in a row
    whose X (and so T) changes: no call may see what an earlier call, or nobody, left there."""
    salr = _salr()
    N = 1000
    x0, w, a_cat, b_cat = _problem(M, K, N, ranks, seed=900 + M)
    rb, rv, ro = oracle.encode(w)
    d = dict(bm=to_dev_u32(rb), v=to_dev_u16(rv), ro=to_dev_u32(ro), a=to_dev_u16(a_cat), b=to_dev_u16(b_cat))
    need = salr.salr_linear_workspace_bytes(M, K, N, sum(ranks))
    ws = torch.randint(0, 256, (need,), dtype=torch.uint8, device=dev())
    for call in range(6):
        x = wl.gaussian_bf16((M, K), 1.0 + call, 7000 + 13 * call + M)
        y = salr.linear(to_dev_u16(x), d["bm"], d["v"], d["ro"], d["a"], d["b"], workspace=ws)
        torch.cuda.synchronize()
        _assert_close(y_to_f64(y), oracle.linear(x, w, a_cat, b_cat), f"M={M} R={sum(ranks)} call {call}")


@pytest.mark.parametrize("M,K,N", [(16, 1024, 2048), (64, 1024, 520), (192, 512, 1000), (300, 1024, 520)])
def test_graph_replays(M, K, N):
    """A captured call (small-batch kernels; large-batch kernels, whose adapter part runs on a forked stream) is
    replayed with new activations in place; the program's own eager work and synchronisations run between replays,
    and every replay is checked."""
    salr = _salr()
    ranks = (32, 16)
    x0, w, a_cat, b_cat = _problem(M, K, N, ranks, seed=4242)
    rb, rv, ro = oracle.encode(w)
    bm, v, rod = to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro)
    a, b = to_dev_u16(a_cat), to_dev_u16(b_cat)
    x_dev = to_dev_u16(x0)
    y = torch.empty((M, N), dtype=x_dev.dtype, device=dev())
    ws = torch.empty(salr.salr_linear_workspace_bytes(M, K, N, sum(ranks)), dtype=torch.uint8, device=dev())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):   # one eager call first, as a capture's warm-up
        salr.salr_sparse_lowrank_linear(x_dev, bm, v, rod, a, b, y, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        salr.salr_sparse_lowrank_linear(x_dev, bm, v, rod, a, b, y, ws)
    for replay in range(5):
        x = wl.gaussian_bf16((M, K), 0.5 + replay, 8100 + replay)
        x_dev.copy_(to_dev_u16(x))
        graph.replay()
        torch.cuda.synchronize()
        _assert_close(y_to_f64(y), oracle.linear(x, w, a_cat, b_cat), f"graph replay {replay}")
        eager = salr.linear(x_dev, bm, v, rod, a, b)   # eager work between the replays, on another workspace
        torch.cuda.synchronize()
        assert torch.equal(eager.view(torch.int16), y.view(torch.int16)), f"replay {replay} differs from eager"


def test_large_batch_calls_back_to_back_share_a_workspace():
    """Calls queued back to back on one stream with ONE workspace and alternating inputs must each give what the same
    call gives alone: nothing of a call may overtake the previous call's MFMA stage, which still reads the workspace."""
    salr = _salr()
    M, K, N = 300, 1024, 520
    xs, ws_, outs = [], [], []
    probs = [_problem(M, K, N, (16, 16), 4200 + i) for i in range(2)]
    enc = []
    for x, w, a_cat, b_cat in probs:
        rb, rv, ro = oracle.encode(w)
        enc.append((to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), to_dev_u16(a_cat), to_dev_u16(b_cat)))
    need = salr.salr_linear_workspace_bytes(M, K, N, 32)
    ws = torch.empty(need, dtype=torch.uint8, device=dev())
    alone = []
    for e in enc:
        alone.append(salr.linear(e[0], e[1], e[2], e[3], e[4], e[5], workspace=ws).clone())
        torch.cuda.synchronize()
    ys = [torch.empty((M, N), dtype=torch.int16, device=dev()) for _ in range(24)]
    for i, y in enumerate(ys):   # no synchronisation in between
        e = enc[i % 2]
        salr.salr_sparse_lowrank_linear(e[0], e[1], e[2], e[3], e[4], e[5], y, ws)
    torch.cuda.synchronize()
    for i, y in enumerate(ys):
        assert torch.equal(y, alone[i % 2].view(torch.int16)), f"call {i}"
    # and against the oracle once
    x, w, a_cat, b_cat = probs[0]
    _assert_close(y_to_f64(ys[0]), oracle.linear(x, w, a_cat, b_cat), "back to back, call 0")
