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


def _plain_on_dequantised(salr, x, rb, codes, scales, ro, nnz, a_cat, b_cat):
    """The layer in two steps through the boundary: dequantise the values, then the plain call on them."""
    v = salr.nf4_dequantize(codes, scales, nnz)
    return salr.linear(x, rb, v, ro, a_cat, b_cat)


@pytest.mark.parametrize("M,K,N,R,permille,seed", [
    (1, 128, 1, 0, 200, 1), (1, 128, 16, 8, 200, 2), (3, 256, 17, 5, 200, 3), (16, 4096, 130, 32, 200, 4),
    (16, 1152, 64, 64, 200, 5), (7, 1024, 300, 0, 200, 6), (17, 2048, 48, 16, 200, 7), (32, 1024, 100, 8, 500, 8),
    (33, 512, 70, 24, 200, 9), (64, 1024, 131, 40, 200, 10), (4, 3968, 33, 12, 0, 11), (5, 640, 40, 4, 950, 12),
    (2, 384, 20, 256, 200, 13), (16, 8192, 40, 64, 200, 14), (9, 14336, 24, 32, 200, 15), (16, 512, 8200, 8, 200, 16),
    (65, 512, 40, 8, 200, 17), (16, 160, 40, 8, 200, 18),
    # large batches: the decode stage of the two-stage path reads the codes (no bf16 copy of the values either)
    (300, 512, 260, 8, 200, 19), (129, 1024, 100, 0, 500, 20), (2048, 256, 192, 16, 200, 21), (200, 4160, 70, 4, 0, 22),
])
def test_qsalr_fused_equals_two_steps(M, K, N, R, permille, seed):
    """Up to 64 tokens on rows of whole chunks the call reads the 4-bit codes itself; it must give, bit for bit, what
    dequantising the values and running the plain layer gives wherever that takes its small-batch streaming kernels
    (the same products enter the same MFMA chain), and that in turn is held to the oracle by test_qsalr_linear and the layer's own parity tests.  Covers one to four m-tiles,
    slices of fewer, exactly and more chunks than a wave keeps in flight, ragged N, every density from all-dense rows
    to 5 %, ranks from 0 to the maximum, two shapes that take the two-step path inside the call, and large batches, where the
    decode stage in front of the dense MFMA stage reads the codes."""
    salr = _salr()
    w = wl.gaussian_bf16((N, K), 0.02, 900 + seed)
    keep = K - (K * permille) // 1000
    w_hat = oracle.mask_topk_rows(w, keep) if permille else w.copy()
    if seed == 12:
        w_hat[3, :] = 0      # an empty row
    x = wl.gaussian_bf16((M, K), 1.0, 950 + seed)
    a_cat = wl.gaussian_bf16((K, R), 0.05, 960 + seed) if R else None
    b_cat = wl.gaussian_bf16((R, N), 0.05, 970 + seed) if R else None
    rb, rv, ro = oracle.encode(w_hat)
    nnz = int(ro[-1])
    codes, scales = salr.nf4_quantize(to_dev_u16(rv))
    xd, rbd, rod = to_dev_u16(x), to_dev_u32(rb), to_dev_u32(ro)
    ad = None if a_cat is None else to_dev_u16(a_cat)
    bd = None if b_cat is None else to_dev_u16(b_cat)
    y = salr.qsalr_linear(xd, rbd, codes, scales, rod, nnz, ad, bd)
    y2 = _plain_on_dequantised(salr, xd, rbd, codes, scales, rod, nnz, ad, bd)
    torch.cuda.synchronize()
    a, b = to_host_u16(y), to_host_u16(y2)
    print(f"[qsalr fused] M{M} K{K} N{N} R{R} p{permille}: {int((a != b).sum())} of {a.size} outputs differ", flush=True)
    if M > 8 and N >= 8192:
        # here the plain layer takes its row-tiled kernel, which splits K differently: equal up to the rounding of
        # the output, not bit for bit
        ya, yb = y_to_f64(y), y_to_f64(y2)
        assert float(np.max(np.abs(ya - yb))) <= 2.0 ** -7 * float(np.max(np.abs(yb)))
    else:
        assert np.array_equal(a, b)


def test_qsalr_fused_against_oracle_and_block_borders():
    """Values chosen so that every scale block has its own magnitude (a wrong block index would be off by orders of
    magnitude), pieces start at every nibble offset, and the result is checked against the oracle directly."""
    salr = _salr()
    M, K, N, R = 8, 512, 96, 16
    rng = np.random.default_rng(77)
    w = wl.gaussian_bf16((N, K), 0.02, 771)
    w_hat = oracle.mask_topk_rows(w, 410)
    # ragged row lengths: drop a different number of further entries per row
    for n_ in range(N):
        drop = rng.choice(np.nonzero(w_hat[n_] & 0x7FFF)[0], size=n_ % 37, replace=False)
        w_hat[n_, drop] = 0
    rb, rv, ro = oracle.encode(w_hat)
    nnz = int(ro[-1])
    # scale block j of the packed values gets magnitude 2^(j % 9 - 4)
    f = oracle.bf16_to_f64(rv) * np.exp2((np.arange(nnz) // 64) % 9 - 4.0)
    rv = wl.f32_to_bf16_bits(f.astype(np.float32))
    rv[(rv & 0x7FFF) == 0] = 0x3C00
    x = wl.gaussian_bf16((M, K), 1.0, 772)
    a_cat = wl.gaussian_bf16((K, R), 0.05, 773)
    b_cat = wl.gaussian_bf16((R, N), 0.05, 774)
    codes_ref, scales_ref = oracle.nf4_quantize(rv)
    w_q = oracle.decode(rb, oracle.nf4_dequantize(codes_ref, scales_ref, nnz), ro, N, K)
    y_ref = oracle.linear(x, w_q, a_cat, b_cat)
    codes, scales = salr.nf4_quantize(to_dev_u16(rv))
    y = salr.qsalr_linear(to_dev_u16(x), to_dev_u32(rb), codes, scales, to_dev_u32(ro), nnz, to_dev_u16(a_cat),
                          to_dev_u16(b_cat))
    torch.cuda.synchronize()
    err = float(np.max(np.abs(y_to_f64(y) - y_ref)))
    scale = float(np.max(np.abs(y_ref)))
    print(f"[qsalr fused, block borders] max|d|={err:.3e} scale={scale:.3e}", flush=True)
    assert err <= 1e-2 * scale
