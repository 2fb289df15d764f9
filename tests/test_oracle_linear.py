"""Pins for the oracle's layer output (paper Sec. 3.2) and SVD residual (Sec. 3.1, Theorem 3).  CPU only."""
import numpy as np
import pytest

import oracle
import salr_workloads as wl


def _f64(bits):
    return oracle.bf16_to_f64(bits)


def _small_problem(M, K, N, ranks, seed, density=0.5, std_ab=0.05):
    rng = np.random.default_rng(seed)
    x = wl.gaussian_bf16((M, K), 1.0, seed + 1)
    w = wl.gaussian_bf16((N, K), 0.02, seed + 2)
    w[rng.random((N, K)) >= density] = 0
    As = [wl.gaussian_bf16((K, r), std_ab, seed + 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), std_ab, seed + 20 + i) for i, r in enumerate(ranks)]
    return x, w, As, Bs


def test_linear_against_pure_python_loops():
    # all four dims different so that a transposed operand cannot pass
    M, K, N, ranks = 3, 11, 5, (2, 1)
    x, w, As, Bs = _small_problem(M, K, N, ranks, 1)
    a_cat, b_cat = wl.concat_adapters(As, Bs)
    R = sum(ranks)
    xf, wf, af, bf = (_f64(t).tolist() for t in (x, w, a_cat, b_cat))
    expect = [[0.0] * N for _ in range(M)]
    for m in range(M):
        t = [sum(xf[m][k] * af[k][r] for k in range(K)) for r in range(R)]
        for n in range(N):
            base = sum(xf[m][k] * wf[n][k] for k in range(K))
            expect[m][n] = base + sum(t[r] * bf[r][n] for r in range(R))
    got = oracle.linear(x, w, a_cat, b_cat)
    np.testing.assert_allclose(got, np.array(expect), rtol=1e-12, atol=1e-15)


def test_linear_special_cases_reduce_to_numpy_matmul():
    M, K, N, ranks = 7, 96, 40, (4, 4)
    x, w, As, Bs = _small_problem(M, K, N, ranks, 2)
    a_cat, b_cat = wl.concat_adapters(As, Bs)
    X, W, A, B = _f64(x), _f64(w), _f64(a_cat), _f64(b_cat)
    # R = 0: plain X What^T
    np.testing.assert_allclose(oracle.linear(x, w, None, None), X @ W.T, rtol=1e-12, atol=1e-14)
    # What = 0: pure low-rank term
    z = np.zeros_like(w)
    np.testing.assert_allclose(oracle.linear(x, z, a_cat, b_cat), (X @ A) @ B, rtol=1e-12, atol=1e-16)
    # p = 0 (dense weight): textbook GEMM plus adapters
    wd = wl.gaussian_bf16((N, K), 0.02, 99)
    np.testing.assert_allclose(oracle.linear(x, wd, a_cat, b_cat), X @ _f64(wd).T + (X @ A) @ B,
                               rtol=1e-12, atol=1e-14)
    # full expression
    np.testing.assert_allclose(oracle.linear(x, w, a_cat, b_cat), X @ W.T + (X @ A) @ B, rtol=1e-12, atol=1e-14)


def test_identity_rows_read_out_the_effective_weight():
    K, N, ranks = 24, 9, (3,)
    _, w, As, Bs = _small_problem(1, K, N, ranks, 3)
    a_cat, b_cat = wl.concat_adapters(As, Bs)
    eye = wl.f32_to_bf16_bits(np.eye(K, dtype=np.float32))
    got = oracle.linear(eye, w, a_cat, b_cat)          # [K, N]: row k = column k of What^T + A B
    np.testing.assert_allclose(got, _f64(w).T + _f64(a_cat) @ _f64(b_cat), rtol=1e-12, atol=1e-16)


def test_concatenated_equals_per_adapter_sum():
    M, K, N, ranks = 4, 64, 48, (8, 8, 4)
    x, w, As, Bs = _small_problem(M, K, N, ranks, 4)
    a_cat, b_cat = wl.concat_adapters(As, Bs)
    assert a_cat.shape == (K, 20) and b_cat.shape == (20, N)
    np.testing.assert_allclose(oracle.linear(x, w, a_cat, b_cat), oracle.linear_per_adapter(x, w, As, Bs),
                               rtol=1e-12, atol=1e-15)


def test_linearity_in_x():
    M, K, N, ranks = 5, 32, 16, (4,)
    x1, w, As, Bs = _small_problem(M, K, N, ranks, 5)
    a_cat, b_cat = wl.concat_adapters(As, Bs)
    # x2 = 2 * x1 is exact in bf16
    x2 = wl.f32_to_bf16_bits(2.0 * wl.bf16_bits_to_f32(x1))
    np.testing.assert_allclose(oracle.linear(x2, w, a_cat, b_cat), 2.0 * oracle.linear(x1, w, a_cat, b_cat),
                               rtol=1e-13, atol=0)


def test_linear_through_the_codec():
    """decode(encode(What)) feeds the same output: the format is transparent to the layer."""
    cfg = wl.CONFIGS["tiny"]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg, rows=64), cfg.keep(500))
    bitmap, values, offsets = oracle.encode(w_hat)
    w_back = oracle.decode(bitmap, values, offsets, 64, cfg.K, use_lut=True)
    x = wl.activations(cfg, 2)
    np.testing.assert_array_equal(oracle.linear(x, w_back, None, None), oracle.linear(x, w_hat, None, None))


@pytest.mark.parametrize("N,K,r", [(512, 512, 8), (512, 512, 16), (256, 384, 16)])
def test_theorem3_svd_residual_bound(N, K, r):
    """||E - E_r||_F^2 <= (1 - r/q) ||E||_F^2 for every matrix; for iid-like residuals the ratio also
    stays above 1 - r (sqrt(N) + sqrt(K))^2 / (N K) (largest singular values of a random matrix)."""
    cfg = wl.CONFIGS["tiny"]
    w = wl.gaussian_bf16((N, K), cfg.std_w, 1234 + N + K)
    w_hat = oracle.mask_topk_rows(w, K - K // 2)
    mse, ratio = oracle.svd_residual_check(w, w_hat, r)
    q = min(N, K)
    assert ratio <= 1.0 - r / q + 1e-12
    assert ratio >= 1.0 - r * (np.sqrt(N) + np.sqrt(K)) ** 2 / (N * K) - 0.01
    # ||E||_F^2 / (NK) is Theorem 1's MSE(p)
    assert abs(mse / oracle.pruning_mse_closed_form(0.5, cfg.std_w) - 1.0) < 0.03


def test_theorem3_equality_for_flat_spectrum():
    # E with all singular values equal (a scaled orthogonal matrix): the bound is attained
    q = 16
    rng = np.random.default_rng(0)
    Q, _ = np.linalg.qr(rng.standard_normal((q, q)))
    s = np.linalg.svd(Q, compute_uv=False)
    for r in (1, 4, 15):
        assert abs(np.sum(s[r:] ** 2) / np.sum(s ** 2) - (1 - r / q)) < 1e-12


def test_residual_adapter_reconstructs_truncated_svd():
    N, K, r = 48, 80, 6
    w = wl.gaussian_bf16((N, K), 0.02, 77)
    w_hat = oracle.mask_topk_rows(w, K // 2)
    A, B = oracle.svd_residual_adapter(w, w_hat, r)
    assert A.shape == (K, r) and B.shape == (r, N)
    E = _f64(w) - _f64(w_hat)
    U, s, Vt = np.linalg.svd(E, full_matrices=False)
    E_r = (U[:, :r] * s[:r]) @ Vt[:r]
    np.testing.assert_allclose(A @ B, E_r.T, atol=1e-12)
    _, ratio = oracle.svd_residual_check(w, w_hat, r)
    assert abs(np.linalg.norm(E - E_r) ** 2 / np.linalg.norm(E) ** 2 - ratio) < 1e-12


def test_f32_to_bf16_hand_values():
    # 1.0 -> 0x3F80; 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80); 1 + 3 * 2^-8 ties to 0x3F82;
    # just above the first tie goes up; -0.0 keeps its sign; the largest fp32 rounds to +inf
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.0, 3.4028234e38],
                 dtype=np.float32)
    np.testing.assert_array_equal(oracle.f32_to_bf16(x), np.array([0x3F80, 0x3F80, 0x3F82, 0x3F81, 0x8000, 0x7F80],
                                                                  dtype=np.uint16))
    assert oracle.f32_to_bf16(np.array([np.nan], dtype=np.float32))[0] & 0x7FFF > 0x7F80


def test_residual_of_a_mask_is_the_pruned_part():
    """Sec. 3.1: W = What + E exactly, E and What have disjoint support, ||E||_F^2 / size is Theorem 1's MSE."""
    N, K = 64, 512
    w = wl.gaussian_bf16((N, K), 0.02, 4711)
    w_hat = oracle.mask_topk_rows(w, K // 2)
    e = oracle.residual(w, w_hat)
    assert e.dtype == np.uint16 and e.shape == w.shape
    kept = (w_hat & 0x7FFF) != 0
    np.testing.assert_array_equal(e[~kept], w[~kept])          # pruned entries move to E bit for bit
    assert not np.any(e[kept] & 0x7FFF)                         # kept entries leave a zero
    np.testing.assert_array_equal(_f64(w_hat) + _f64(e), _f64(w))
    mse = float(np.sum(_f64(e) ** 2)) / e.size
    assert abs(mse / oracle.pruning_mse_closed_form(0.5, 0.02) - 1.0) < 0.05


def test_residual_hand_values():
    # bf16 patterns: 1.0 = 0x3F80, 0.5 = 0x3F00, 2^-8 = 0x3B80, 255/256 = 0x3F7F, -1.5 = 0xBFC0, 2.5 = 0x4020
    w = np.array([[0x3F80, 0x3F80, 0x3F00, 0xBFC0]], dtype=np.uint16)
    h = np.array([[0x3F00, 0x3B80, 0x3F00, 0x3F80]], dtype=np.uint16)
    # 1 - 0.5 = 0.5; 1 - 2^-8 = 255/256; 0.5 - 0.5 = +0; -1.5 - 1 = -2.5
    np.testing.assert_array_equal(oracle.residual(w, h), np.array([[0x3F00, 0x3F7F, 0x0000, 0xC020]], dtype=np.uint16))


def test_concat_adapters_is_the_sum_over_adapters():
    """Sec. 3.2 on small integers (every product and sum exact in fp64): (x A_cat) B_cat = sum_i (x A_i) B_i, and the
    blocks sit where the definition puts them."""
    rng = np.random.default_rng(5)
    K, N, ranks = 7, 5, (1, 3, 2)
    As = [rng.integers(-4, 5, (K, r)).astype(np.float64) for r in ranks]
    Bs = [rng.integers(-4, 5, (r, N)).astype(np.float64) for r in ranks]
    a_cat, b_cat = oracle.concat_adapters(As, Bs)
    assert a_cat.shape == (K, 6) and b_cat.shape == (6, N)
    np.testing.assert_array_equal(a_cat[:, 1:4], As[1])
    np.testing.assert_array_equal(b_cat[4:6, :], Bs[2])
    x = rng.integers(-3, 4, (4, K)).astype(np.float64)
    np.testing.assert_array_equal((x @ a_cat) @ b_cat, sum((x @ a) @ b for a, b in zip(As, Bs)))
    # and on bf16 patterns it is a bit copy, equal to the input generator's stacking
    A16 = [wl.gaussian_bf16((K, r), 0.01, 30 + i) for i, r in enumerate(ranks)]
    B16 = [wl.gaussian_bf16((r, N), 0.01, 40 + i) for i, r in enumerate(ranks)]
    a1, b1 = oracle.concat_adapters(A16, B16)
    a2, b2 = wl.concat_adapters(A16, B16)
    np.testing.assert_array_equal(a1, a2)
    np.testing.assert_array_equal(b1, b2)


def test_backward_is_the_adjoint_of_the_forward():
    """<dY, Y(X)> = <dX, X>;  <dY, Y(A + dA') - Y(A)> = <dA, dA'>;  the same for B.  The forward pass is the oracle's C
    code, so the numpy products in linear_backward are pinned by something that is not numpy."""
    M, K, N, ranks = 5, 64, 12, (3, 2)
    x, w, a_cat, b_cat = (wl.gaussian_bf16((M, K), 1.0, 1), wl.gaussian_bf16((N, K), 0.5, 2), None, None)
    w_hat = oracle.mask_topk_rows(w, K // 2)
    As = [wl.gaussian_bf16((K, r), 0.5, 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), 0.5, 20 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = wl.concat_adapters(As, Bs)
    dy = wl.gaussian_bf16((M, N), 1.0, 3)
    dx, da, db = oracle.linear_backward(x, dy, w_hat, a_cat, b_cat)
    assert dx.shape == (M, K) and da.shape == a_cat.shape and db.shape == b_cat.shape
    y = oracle.linear(x, w_hat, a_cat, b_cat)
    assert abs(np.sum(_f64(dy) * y) - np.sum(dx * _f64(x))) < 1e-9 * np.sum(np.abs(_f64(dy) * y))
    # directions that are themselves bf16 patterns, so that A + dA' is exactly representable as an oracle input is not
    # needed: Y is linear in A and in B, so Y(dA', B) - Y(0, B) = (X dA') B
    a2 = wl.gaussian_bf16(a_cat.shape, 0.5, 30)
    y_dir = oracle.linear(x, np.zeros_like(w_hat), a2, b_cat)
    assert abs(np.sum(_f64(dy) * y_dir) - np.sum(da * _f64(a2))) < 1e-9 * np.sum(np.abs(_f64(dy) * y_dir))
    b2 = wl.gaussian_bf16(b_cat.shape, 0.5, 31)
    y_dir = oracle.linear(x, np.zeros_like(w_hat), a_cat, b2)
    assert abs(np.sum(_f64(dy) * y_dir) - np.sum(db * _f64(b2))) < 1e-9 * np.sum(np.abs(_f64(dy) * y_dir))


def test_backward_against_python_loops():
    M, K, N, R = 2, 32, 3, 2
    x, dy = wl.gaussian_bf16((M, K), 1.0, 4), wl.gaussian_bf16((M, N), 1.0, 5)
    w_hat = oracle.mask_topk_rows(wl.gaussian_bf16((N, K), 0.5, 6), 10)
    a, b = wl.gaussian_bf16((K, R), 0.5, 7), wl.gaussian_bf16((R, N), 0.5, 8)
    X, dY, W, A, B = (_f64(t) for t in (x, dy, w_hat, a, b))
    dx, da, db = oracle.linear_backward(x, dy, w_hat, a, b)
    for m in range(M):
        for k in range(K):
            s = sum(dY[m, n] * W[n, k] for n in range(N))
            s += sum(sum(dY[m, n] * B[r, n] for n in range(N)) * A[k, r] for r in range(R))
            assert abs(dx[m, k] - s) < 1e-12
    for k in range(K):
        for r in range(R):
            assert abs(da[k, r] - sum(X[m, k] * sum(dY[m, n] * B[r, n] for n in range(N)) for m in range(M))) < 1e-12
    for r in range(R):
        for n in range(N):
            assert abs(db[r, n] - sum(sum(X[m, k] * A[k, r] for k in range(K)) * dY[m, n] for m in range(M))) < 1e-12
    only_dx, none_a, none_b = oracle.linear_backward(x, dy, w_hat, None, None)
    assert none_a is None and none_b is None
    np.testing.assert_allclose(only_dx, dY @ W, atol=1e-12)
