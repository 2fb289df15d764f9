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
