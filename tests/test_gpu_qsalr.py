"""GPU parity for QSALR (paper Sec. 4, 20 % sparsity + NF4 coding of the packed values) through the C boundary:
codes, scales and dequantised values bit for bit against the oracle (every decision is an fp32 comparison both sides
take alike); the layer on the quantised weight within max |Y - Y_ref| <= 1e-2 * max |Y_ref| of the fp64 oracle
evaluated on the oracle's own dequantised weight."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import dev, to_dev_u16, to_dev_u32, to_host_u16, y_to_f64

pytestmark = pytest.mark.gpu


def _salr():
    import paper_2601_16991_amd as salr
    return salr


def _values(n, seed, std=0.02):
    v = wl.gaussian_bf16((n,), std, seed)
    v[(v & 0x7FFF) == 0] = 0x3C00
    return v


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 128, 1000, 4097, 64 * 5000 + 33])
def test_quantize_dequantize_bit_exact(n):
    salr = _salr()
    v = _values(n, 100 + n)
    codes_ref, scales_ref = oracle.nf4_quantize(v)
    codes, scales = salr.nf4_quantize(to_dev_u16(v))
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), codes_ref)
    assert np.array_equal(to_host_u16(scales), scales_ref)
    back = salr.nf4_dequantize(codes, scales, n)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_u16(back), oracle.nf4_dequantize(codes_ref, scales_ref, n))


def test_quantize_special_values():
    """Magnitudes spread over many binades inside one block, values on and next to the boundaries, zeros and -0.0."""
    salr = _salr()
    lv = oracle.nf4_codebook()
    mids = 0.5 * (lv[:-1] + lv[1:])
    blocks = []
    for scale in (1.0, 0.0123, 3.0e-5, 257.0):
        vals = np.concatenate([lv * scale, mids * scale, mids * scale * 1.01, mids * scale * 0.99, [0.0, -0.0, scale]])
        blocks.append(np.resize(vals.astype(np.float32), 64))
    v = wl.f32_to_bf16_bits(np.concatenate(blocks))
    v[70] = 0x8000
    codes_ref, scales_ref = oracle.nf4_quantize(v)
    codes, scales = salr.nf4_quantize(to_dev_u16(v))
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), codes_ref)
    assert np.array_equal(to_host_u16(scales), scales_ref)
    z = np.zeros(130, dtype=np.uint16)
    codes, scales = salr.nf4_quantize(to_dev_u16(z))
    torch.cuda.synchronize()
    cr, sr = oracle.nf4_quantize(z)
    assert np.array_equal(codes.cpu().numpy(), cr) and np.array_equal(to_host_u16(scales), sr)


@pytest.mark.parametrize("M,K,N,ranks,permille", [
    (1, 512, 100, (8,), 200), (16, 1024, 520, (16, 16), 200), (40, 2048, 132, (4,), 200), (300, 512, 260, (8, 8), 200),
    (8, 14336, 48, (64,), 200), (5, 256, 64, (), 500),
])
def test_qsalr_linear(M, K, N, ranks, permille):
    salr = _salr()
    seed = 40 * M + K + N
    w = wl.gaussian_bf16((N, K), 0.02, seed)
    w_hat = oracle.mask_topk_rows(w, K - (K * permille) // 1000)
    x = wl.gaussian_bf16((M, K), 1.0, seed + 1)
    As = [wl.gaussian_bf16((K, r), 0.05, seed + 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), 0.05, seed + 20 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = wl.concat_adapters(As, Bs) if ranks else (None, None)
    rb, rv, ro = oracle.encode(w_hat)
    nnz = int(ro[-1])
    codes_ref, scales_ref = oracle.nf4_quantize(rv)
    # the weight the quantised format stands for, by the oracle alone
    w_q = oracle.decode(rb, oracle.nf4_dequantize(codes_ref, scales_ref, nnz), ro, N, K)
    y_ref = oracle.linear(x, w_q, a_cat, b_cat)
    codes, scales = salr.nf4_quantize(to_dev_u16(rv))
    y = salr.qsalr_linear(to_dev_u16(x), to_dev_u32(rb), codes, scales, to_dev_u32(ro), nnz,
                          None if a_cat is None else to_dev_u16(a_cat), None if b_cat is None else to_dev_u16(b_cat))
    torch.cuda.synchronize()
    err = float(np.max(np.abs(y_to_f64(y) - y_ref)))
    scale = float(np.max(np.abs(y_ref)))
    print(f"[qsalr] M{M} K{K} N{N} R{sum(ranks)} p{permille}: max|d|={err:.3e} scale={scale:.3e}", flush=True)
    assert err <= 1e-2 * scale
    # and the quantisation itself is the small perturbation it should be: relative Frobenius error of the weight
    e = np.linalg.norm(oracle.bf16_to_f64(w_q) - oracle.bf16_to_f64(w_hat)) / np.linalg.norm(oracle.bf16_to_f64(w_hat))
    assert e < 0.15
