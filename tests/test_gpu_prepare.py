"""GPU parity: salr_residual and salr_concat_adapters through the C boundary vs the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import dev, to_dev_u16, to_host_u16

pytestmark = pytest.mark.gpu


def _salr():
    import paper_2601_16991_amd as salr
    return salr


@pytest.mark.parametrize("N,K", [(1, 1), (3, 37), (64, 512), (129, 1000), (257, 4096)])
def test_residual_of_masks(N, K):
    salr = _salr()
    w = wl.gaussian_bf16((N, K), 0.02, 100 + N + K)
    w_hat = oracle.mask_topk_rows(w, K - K // 2)
    e = salr.residual(to_dev_u16(w), to_dev_u16(w_hat))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host_u16(e), oracle.residual(w, w_hat))


def test_residual_of_unrelated_matrices_rounds_like_the_oracle():
    salr = _salr()
    rng = np.random.default_rng(9)
    w = rng.integers(0, 1 << 16, (77, 333)).astype(np.uint16)     # every pattern: NaN, Inf, denormals, both zeros
    h = rng.integers(0, 1 << 16, (77, 333)).astype(np.uint16)
    e = to_host_u16(salr.residual(to_dev_u16(w), to_dev_u16(h)))
    ref = oracle.residual(w, h)
    nan = (ref & 0x7FFF) > 0x7F80
    np.testing.assert_array_equal(e[~nan], ref[~nan])
    assert np.all((e[nan] & 0x7FFF) > 0x7F80)                      # a NaN stays a NaN; its payload is not compared


def test_residual_empty():
    salr = _salr()
    e = salr.residual(torch.empty((0, 64), dtype=torch.int16, device=dev()), torch.empty((0, 64), dtype=torch.int16, device=dev()))
    assert e.shape == (0, 64)


@pytest.mark.parametrize("K,N,ranks", [(64, 96, (8,)), (100, 52, (1, 3, 2)), (4096, 1024, (32, 16, 64)),
                                      (33, 17, (4, 0, 5)), (256, 264, tuple([2] * 19))])
def test_concat_adapters(K, N, ranks):
    salr = _salr()
    As = [wl.gaussian_bf16((K, r), 0.01, 300 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), 0.01, 400 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = salr.concat_adapters([to_dev_u16(a) for a in As], [to_dev_u16(b) for b in Bs])
    torch.cuda.synchronize()
    ra, rb = oracle.concat_adapters(As, Bs)
    np.testing.assert_array_equal(to_host_u16(a_cat), ra)
    np.testing.assert_array_equal(to_host_u16(b_cat), rb)


def test_concat_feeds_the_linear():
    """The concatenation built on the GPU gives the layer output of the per-adapter sum (Sec. 3.2)."""
    salr = _salr()
    M, K, N, ranks = 8, 256, 192, (16, 8, 24)
    x = wl.gaussian_bf16((M, K), 1.0, 1)
    w = wl.gaussian_bf16((N, K), 0.02, 2)
    w_hat = oracle.mask_topk_rows(w, K // 2)
    As = [wl.gaussian_bf16((K, r), 0.05, 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), 0.05, 20 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = salr.concat_adapters([to_dev_u16(a) for a in As], [to_dev_u16(b) for b in Bs])
    bm, v, ro = salr.encode(to_dev_u16(w_hat))
    y = salr.linear(to_dev_u16(x), bm, v, ro, a_cat, b_cat)
    torch.cuda.synchronize()
    from gpu_util import y_to_f64
    ref = oracle.linear_per_adapter(x, w_hat, As, Bs)
    assert np.max(np.abs(y_to_f64(y) - ref)) <= 1e-2 * np.max(np.abs(ref))


# ---------------------------------------------------------------------------------------------------
# salr_residual_adapter (Sec. 3.1).  The pair (A_res, B_res) is not unique; its product is compared: the Frobenius
# error against E must stay within a stated factor of the optimum ||E - E_r||_F (Eckart-Young, from the oracle's
# fp64 SVD), and the singular values found must match the leading ones of E.
# ---------------------------------------------------------------------------------------------------
def _f64(bits):
    return oracle.bf16_to_f64(bits)


def _run_adapter(e_bits, r, oversample, iterations, seed=0):
    salr = _salr()
    N, K = e_bits.shape
    omega = np.random.default_rng(seed).standard_normal((K, r + oversample)).astype(np.float32)
    a, b, s = salr.residual_adapter(to_dev_u16(e_bits), r, torch.from_numpy(omega).to(dev()), iterations)
    torch.cuda.synchronize()
    return to_host_u16(a), to_host_u16(b), s.cpu().numpy().astype(np.float64)


def _optimum(e_bits, r):
    sv = np.linalg.svd(_f64(e_bits), compute_uv=False)
    return sv, float(np.sqrt(np.sum(sv[r:] ** 2)))


def test_residual_adapter_recovers_an_exactly_low_rank_matrix():
    """Rank 3, small integers (exact in bf16): the pair reproduces E up to the bf16 rounding of its factors, the
    fourth singular value comes out as (numerically) zero and its column / row as zeros."""
    rng = np.random.default_rng(3)
    N, K = 128, 96
    E = sum(np.outer(rng.integers(-2, 3, N), rng.integers(-2, 3, K)) for _ in range(3)).astype(np.float32)
    e_bits = oracle.f32_to_bf16(E)
    np.testing.assert_array_equal(_f64(e_bits), E)
    a, b, s = _run_adapter(e_bits, 4, 4, 1)
    sv, _ = _optimum(e_bits, 4)
    err = np.linalg.norm(E - (_f64(a) @ _f64(b)).T)
    print(f"[adapter] low rank: err/||E|| = {err / np.linalg.norm(E):.2e}, sigma = {s}, exact = {sv[:4]}", flush=True)
    assert err <= 1e-2 * np.linalg.norm(E)
    np.testing.assert_allclose(s[:3], sv[:3], rtol=2e-3)
    assert s[3] <= 2e-3 * sv[0]


@pytest.mark.parametrize("N,K,r,oversample,iters,decay", [(256, 192, 8, 8, 2, 0.9), (192, 320, 16, 8, 2, 0.9),
                                                          (512, 256, 32, 16, 2, 0.9), (256, 256, 64, 16, 2, 0.9),
                                                          (384, 512, 100, 28, 3, 0.97)])
def test_residual_adapter_on_a_decaying_spectrum(N, K, r, oversample, iters, decay):
    """sigma_i = decay^i (rounded to bf16 entries; sigma_r stays above 1e-3 sigma_1: the l x l eigenproblem is solved
    on Z^T Z in fp32, which resolves singular values far below that only roughly): after two or three rounds the error is within 2 % of the optimum (plus the
    bf16 rounding of the two factors) and the singular values within 1 %."""
    rng = np.random.default_rng(N + K + r)
    q = min(N, K)
    U, _ = np.linalg.qr(rng.standard_normal((N, q)))
    V, _ = np.linalg.qr(rng.standard_normal((K, q)))
    e_bits = oracle.f32_to_bf16(((U * (decay ** np.arange(q))) @ V.T).astype(np.float32))
    a, b, s = _run_adapter(e_bits, r, oversample, iters)
    assert a.shape == (K, r) and b.shape == (r, N)
    sv, opt = _optimum(e_bits, r)
    err = np.linalg.norm(_f64(e_bits) - (_f64(a) @ _f64(b)).T)
    print(f"[adapter] decaying N={N} K={K} r={r}: err/opt = {err / opt:.4f}, max sigma dev = "
          f"{np.max(np.abs(s / sv[:r] - 1)):.2e}", flush=True)
    assert err >= opt * (1 - 1e-6)
    # the method's share: 2 % over the optimum; the outputs' share: both factors are rounded to bf16 (2^-9 relative
    # each, so 2^-8 on every term of the product, i.e. at most 2^-8 ||E_r||_F on the whole)
    rounding = 2.0 ** -8 * np.sqrt(np.sum(sv[:r] ** 2))
    assert err <= np.hypot(1.02 * opt, rounding)
    np.testing.assert_allclose(s, sv[:r], rtol=1e-2)
    assert np.all(np.diff(s) <= 1e-6 * s[0])


def test_residual_adapter_smallest_sizes_and_full_rank():
    """32 x 32 (the smallest legal size) with a sketch as wide as the matrix: the range finder spans everything, the
    result is the exact truncated SVD up to rounding; also a sketch width that is not a multiple of 16."""
    rng = np.random.default_rng(11)
    e_bits = oracle.f32_to_bf16(rng.standard_normal((32, 32)).astype(np.float32))
    for r, over in ((4, 28), (5, 6)):
        a, b, s = _run_adapter(e_bits, r, over, 3)
        sv, opt = _optimum(e_bits, r)
        err = np.linalg.norm(_f64(e_bits) - (_f64(a) @ _f64(b)).T)
        print(f"[adapter] 32x32 r={r} l={r + over}: err/opt = {err / opt:.4f}", flush=True)
        assert err >= opt * (1 - 1e-6)
        rounding = 2.0 ** -8 * np.sqrt(np.sum(sv[:r] ** 2))
        assert err <= np.hypot((1.001 if over == 28 else 1.10) * opt, rounding)
        if over == 28:
            np.testing.assert_allclose(s, sv[:r], rtol=1e-3)


def test_residual_adapter_on_a_pruning_residual():
    """E = W - What of a Gaussian W at p = 0.5 (the workload of this build: a flat, Marchenko-Pastur-like spectrum, the
    hardest case for a subspace iteration).  The captured energy ||E||^2 - err^2 reaches 90 % of the optimum's after
    four rounds, and Theorem 3's bound holds for the pair."""
    N, K, r = 512, 512, 16
    w = wl.gaussian_bf16((N, K), 0.02, 99)
    e_bits = oracle.residual(w, oracle.mask_topk_rows(w, K // 2))
    a, b, s = _run_adapter(e_bits, r, 16, 4)
    sv, opt = _optimum(e_bits, r)
    E = _f64(e_bits)
    total = np.linalg.norm(E) ** 2
    err = np.linalg.norm(E - (_f64(a) @ _f64(b)).T)
    captured, best = total - err ** 2, total - opt ** 2
    print(f"[adapter] pruning residual: captured/best = {captured / best:.4f}, err/opt = {err / opt:.4f}", flush=True)
    assert err >= opt * (1 - 1e-6)
    assert captured >= 0.90 * best
    assert err ** 2 <= (1 - r / min(N, K)) * total          # Theorem 3's bound, which the exact E_r satisfies a fortiori


def test_residual_adapter_then_linear_adds_the_correction():
    """Appending the pair to the adapters adds x E_r^T to the layer output (Sec. 3.1 with Sec. 3.2)."""
    salr = _salr()
    M, N, K, r = 8, 256, 192, 8
    rng = np.random.default_rng(8)
    U, _ = np.linalg.qr(rng.standard_normal((N, K)))
    V, _ = np.linalg.qr(rng.standard_normal((K, K)))
    e_bits = oracle.f32_to_bf16((0.5 * (U * (0.8 ** np.arange(K))) @ V.T).astype(np.float32))
    a, b, _ = _run_adapter(e_bits, r, 8, 2)
    x = wl.gaussian_bf16((M, K), 1.0, 5)
    zero = np.zeros((N, K), dtype=np.uint16)
    bm, v, ro = salr.encode(to_dev_u16(zero))
    y = salr.linear(to_dev_u16(x), bm, v, ro, to_dev_u16(a), to_dev_u16(b))
    torch.cuda.synchronize()
    from gpu_util import y_to_f64
    Ue, se, Vte = np.linalg.svd(_f64(e_bits), full_matrices=False)
    ref = _f64(x) @ ((Ue[:, :r] * se[:r]) @ Vte[:r]).T
    assert np.max(np.abs(y_to_f64(y) - ref)) <= 2e-2 * np.max(np.abs(ref))


def test_residual_adapter_full_size_properties():
    """q_proj size (4096 x 4096, p = 0.5, r = 32), where the fp64 SVD is too slow to serve as a check: properties that
    hold at any size.  The pair is (up to rounding) an orthogonal projection of E, so ||E - P||^2 = ||E||^2 - ||P||^2
    and ||P||^2 = sum sigma_k^2; Theorem 3's bound; singular values descending and inside the Marchenko-Pastur
    range of a residual with iid entries of variance MSE(p) sigma_w^2."""
    N = K = 4096
    r = 32
    cfg = wl.CONFIGS["llama3_8b_q_proj"]
    w = wl.dense_weight(cfg)
    e_bits = oracle.residual(w, oracle.mask_topk_rows(w, K // 2))
    a, b, s = _run_adapter(e_bits, r, 16, 2)
    E = _f64(e_bits)
    P = (_f64(a) @ _f64(b)).T
    total, perr, pnorm = np.linalg.norm(E) ** 2, np.linalg.norm(E - P) ** 2, np.linalg.norm(P) ** 2
    print(f"[adapter] 4096^2: captured {1 - perr / total:.4%}, ||P||^2 / sum sigma^2 = {pnorm / np.sum(s ** 2):.4f}", flush=True)
    assert abs(pnorm / np.sum(s ** 2) - 1) < 1e-2
    assert abs((total - perr) / pnorm - 1) < 2e-2
    assert perr <= (1 - r / N) * total
    assert np.all(np.diff(s) <= 0)
    edge = np.sqrt(oracle.pruning_mse_closed_form(0.5, cfg.std_w)) * (np.sqrt(N) + np.sqrt(K))
    assert 0.8 * edge < s[-1] <= s[0] < 1.05 * edge
