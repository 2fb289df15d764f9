"""GPU parity on seeded random shapes: the layer (plain call, prepared call, QSALR call) through the C boundary against
the fp64 CPU oracle, max |Y - Y_ref| <= 1e-2 * max |Y_ref|.  The hand-picked cases of the other files aim at each
kernel's edges; these draw batch size, row length, row count, rank and density at random over the ranges where the
dispatch changes kernels, so that a combination nobody thought of still gets checked."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import to_dev_u16, to_dev_u32, y_to_f64

pytestmark = pytest.mark.gpu
REL_TOL = 1e-2


def _draw(seed):
    rng = np.random.default_rng(10_000 + seed)
    M = int(rng.choice([1, 2, 5, 8, 9, 16, 17, 31, 32, 33, 48, 64, 65, 100, 128, 129, 200, 300]))
    kind = int(rng.integers(0, 4))
    if kind == 0:
        K = 128 * int(rng.integers(1, 40))                 # whole chunks
    elif kind == 1:
        K = 32 * int(rng.integers(1, 70))                  # any whole number of bitmap words
    elif kind == 2:
        K = int(rng.choice([4096, 8192, 12288, 14336]))    # the row lengths of the workloads
    else:
        K = 64 * int(rng.integers(1, 50))
    big_k = K >= 4096
    N = int(rng.integers(1, 260 if big_k else 1200))
    if rng.random() < 0.15:
        N = int(rng.choice([8192 + 16, 8200, 9000])) if K <= 1024 else N   # many rows: the row-tiled kernel from 9 tokens
    R = int(rng.choice([0, 1, 4, 8, 16, 32, 33, 64, 100]))
    density = float(rng.choice([0.05, 0.3, 0.5, 0.5, 0.7, 0.8, 1.0]))
    return M, K, N, R, density


@pytest.mark.parametrize("seed", range(48))
def test_random_shape(seed):
    import paper_2601_16991_amd as salr
    M, K, N, R, density = _draw(seed)
    rng = np.random.default_rng(20_000 + seed)
    x = wl.gaussian_bf16((M, K), 1.0, 30_000 + seed)
    w = wl.gaussian_bf16((N, K), 0.02, 40_000 + seed)
    w[rng.random((N, K)) >= density] = 0
    a_cat = wl.gaussian_bf16((K, R), 0.01, 50_000 + seed) if R else None
    b_cat = wl.gaussian_bf16((R, N), 0.01, 60_000 + seed) if R else None
    print(f"[random] seed {seed}: M{M} K{K} N{N} R{R} density {density}", flush=True)
    rb, rv, ro = oracle.encode(w)
    nnz = int(ro[-1])
    xd, bm, v, rod = to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro)
    a = None if a_cat is None else to_dev_u16(a_cat)
    b = None if b_cat is None else to_dev_u16(b_cat)
    y_ref = oracle.linear(x, w, a_cat, b_cat)
    scale = float(np.max(np.abs(y_ref)))

    y = salr.linear(xd, bm, v, rod, a, b)
    table = salr.build_slice_table(bm, rod, K)
    y_t = salr.linear_prepared(xd, bm, v, rod, table, a, b)
    torch.cuda.synchronize()
    for name, got in (("plain", y), ("prepared", y_t)):
        err = float(np.max(np.abs(y_to_f64(got) - y_ref)))
        print(f"[random] {name}: max|d|={err:.3e} scale={scale:.3e}", flush=True)
        assert err <= REL_TOL * scale + 1e-30, name

    if nnz:
        # QSALR on the same weight: against the oracle's layer on the oracle's dequantised values
        codes_ref, scales_ref = oracle.nf4_quantize(rv)
        w_q = oracle.decode(rb, oracle.nf4_dequantize(codes_ref, scales_ref, nnz), ro, N, K)
        yq_ref = oracle.linear(x, w_q, a_cat, b_cat)
        codes, scales = salr.nf4_quantize(v)
        yq = salr.qsalr_linear(xd, bm, codes, scales, rod, nnz, a, b)
        torch.cuda.synchronize()
        qscale = float(np.max(np.abs(yq_ref)))
        err = float(np.max(np.abs(y_to_f64(yq) - yq_ref)))
        print(f"[random] qsalr: max|d|={err:.3e} scale={qscale:.3e}", flush=True)
        assert err <= REL_TOL * qscale + 1e-30, "qsalr"
