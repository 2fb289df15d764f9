"""GPU parity at full size for every layer shape / batch size the workload list names (see salr_workloads.CONFIGS),
in the launch configuration bench.py times: salr_sparse_lowrank_linear through the C boundary vs the fp64 CPU oracle.

Batches the oracle finishes in seconds are compared element by element on all outputs; larger batches on a fixed sample
of rows of X across all N outputs (every output column, hence every weight row and every tile column, is covered; the
sampled rows sit in the first, a middle and the last row tile).

Bar: max |Y - Y_ref| <= 1e-2 * max |Y_ref| (bf16 inputs, fp32 accumulation, bf16 output)."""
import functools

import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import to_dev_u16, to_dev_u32, to_host_u16

pytestmark = pytest.mark.gpu

REL_TOL = 1e-2
FULL_ORACLE_MAX_M = 64       # above this the oracle checks sampled rows


@functools.lru_cache(maxsize=1)
def _layer(name, permille):
    """Masked weight, its encoding on the device and the adapters of one layer; one layer is kept at a time."""
    cfg = wl.CONFIGS[name]
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(permille))
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    rb, rv, ro = oracle.encode(w_hat)
    assert int(ro[-1]) == cfg.N * cfg.keep(permille)
    d = (to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), to_dev_u16(a_cat), to_dev_u16(b_cat))
    return cfg, w_hat, a_cat, b_cat, d


def _cases():
    out = []
    for name, cfg in wl.CONFIGS.items():
        for permille in cfg.sparsity_permille:
            for M in cfg.Ms:
                out.append(pytest.param(name, permille, M, id=f"{name}-p{permille}-M{M}"))
    return out


@pytest.mark.parametrize("name,permille,M", _cases())
def test_config_full_size(name, permille, M):
    import paper_2601_16991_amd as salr
    cfg, w_hat, a_cat, b_cat, d = _layer(name, permille)
    x = wl.activations(cfg, M)
    print(f"[configs] {name} p={permille} M={M}: launching", flush=True)
    y = salr.linear(to_dev_u16(x), *d)
    torch.cuda.synchronize()
    y = to_host_u16(y)
    assert ((y & 0x7F80) != 0x7F80).all(), "non-finite output"
    if M <= FULL_ORACLE_MAX_M:
        rows = np.arange(M)
    else:
        rows = np.unique(np.array([0, 15, 16, 255, 256, M // 2 + 1, M - 2, M - 1]))
    y_ref = oracle.linear(np.ascontiguousarray(x[rows]), w_hat, a_cat, b_cat)
    scale = float(np.max(np.abs(y_ref)))
    err = float(np.max(np.abs(wl.bf16_bits_to_f32(y[rows]).astype(np.float64) - y_ref)))
    print(f"[configs] {name} p={permille} M={M}: {len(rows)} of {M} rows checked, max|d|={err:.3e} scale={scale:.3e} "
          f"rel={err / scale:.2e}", flush=True)
    assert err <= REL_TOL * scale, f"{name} p={permille} M={M}: {err} > {REL_TOL} * {scale}"
