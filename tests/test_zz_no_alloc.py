"""GPU test of salr_sparse_lowrank_linear_noalloc (the entry point for callers that cannot allocate): through the C
boundary, against salr_sparse_lowrank_linear on the same inputs (bit for bit: the kernels are the same, only the
scratch memory differs) and against the fp64 oracle (max |Y - Y_ref| <= 1e-2 * max |Y_ref|), on two calls in a row,
the second with a smaller input, so that whatever the first call left in the library's scratch array is there when
the second one runs."""
import numpy as np
import pytest
import torch

import oracle
import salr_workloads as wl
from gpu_util import dev, to_dev_u16, to_dev_u32, y_to_f64

pytestmark = pytest.mark.gpu

REL_TOL = 1e-2


def _problem(M, K, N, ranks, seed):
    rng = np.random.default_rng(seed)
    x = wl.gaussian_bf16((M, K), 1.0, seed + 1)
    w = wl.gaussian_bf16((N, K), 0.02, seed + 2)
    w[rng.random((N, K)) >= 0.5] = 0
    As = [wl.gaussian_bf16((K, r), 0.05, seed + 10 + i) for i, r in enumerate(ranks)]
    Bs = [wl.gaussian_bf16((r, N), 0.05, seed + 20 + i) for i, r in enumerate(ranks)]
    a_cat, b_cat = wl.concat_adapters(As, Bs)
    return x, w, a_cat, b_cat


def _both(salr, x, w, a_cat, b_cat):
    rb, rv, ro = oracle.encode(w)
    d = (to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), to_dev_u16(a_cat), to_dev_u16(b_cat))
    y_ws = salr.linear(*d)                              # the existing entry point, workspace from torch
    y_na = torch.empty_like(y_ws)
    salr.salr_sparse_lowrank_linear_noalloc(*d, y_na)   # the library's own scratch array
    torch.cuda.synchronize()
    return y_ws, y_na


# (first call, second, smaller call): small-batch kernel with split-K partials of T; row-tiled kernel with partials
# of T and of Y (K split over workgroups); a layer-sized first call
@pytest.mark.parametrize("first,second", [
    ((16, 1024, 520, (16, 16)), (3, 256, 100, (8,))),
    ((64, 2048, 260, (32, 32)), (40, 512, 132, (4,))),
    ((16, 4096, 4096, (16, 16)), (1, 4096, 4096, (16, 16))),
])
def test_noalloc_matches_workspace_call_twice_in_a_row(first, second):
    import paper_2601_16991_amd as salr
    for call, (M, K, N, ranks) in enumerate((first, second)):
        assert 0 < salr.salr_linear_workspace_bytes(M, K, N, sum(ranks)) <= salr.NOALLOC_SCRATCH_BYTES
        x, w, a_cat, b_cat = _problem(M, K, N, ranks, 77 + 5 * M + N)
        print(f"[noalloc] call {call}: M{M} K{K} N{N} R{sum(ranks)}", flush=True)
        y_ws, y_na = _both(salr, x, w, a_cat, b_cat)
        assert torch.equal(y_ws, y_na), f"call {call}: differs from salr_sparse_lowrank_linear"
        y_ref = oracle.linear(x, w, a_cat, b_cat)
        err = float(np.max(np.abs(y_to_f64(y_na) - y_ref)))
        scale = float(np.max(np.abs(y_ref)))
        print(f"[noalloc] call {call}: max|d|={err:.3e} scale={scale:.3e}", flush=True)
        assert err <= REL_TOL * scale


def test_noalloc_large_batch_takes_the_kernel_without_a_decoded_copy():
    """A large batch whose preferred workspace (a decoded copy of the weight) is beyond the fixed array runs the fused
    kernel on the adapter intermediates alone; against the workspace call given that same least size, and the oracle."""
    import paper_2601_16991_amd as salr
    M, K, N, ranks = 300, 8192, 1200, (16, 16)
    R = sum(ranks)
    assert salr.salr_linear_workspace_bytes(M, K, N, R) > salr.NOALLOC_SCRATCH_BYTES
    least = salr.salr_linear_workspace_bytes_min(M, K, N, R)
    assert 0 < least <= salr.NOALLOC_SCRATCH_BYTES
    x, w, a_cat, b_cat = _problem(M, K, N, ranks, 4321)
    rb, rv, ro = oracle.encode(w)
    d = (to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), to_dev_u16(a_cat), to_dev_u16(b_cat))
    y_ws = salr.linear(*d, workspace=torch.empty(least, dtype=torch.uint8, device=dev()))
    y_na = torch.empty_like(y_ws)
    salr.salr_sparse_lowrank_linear_noalloc(*d, y_na)
    torch.cuda.synchronize()
    assert torch.equal(y_ws, y_na)
    y_ref = oracle.linear(x, w, a_cat, b_cat)
    assert float(np.max(np.abs(y_to_f64(y_na) - y_ref))) <= REL_TOL * float(np.max(np.abs(y_ref)))


def test_noalloc_refuses_sizes_beyond_its_scratch():
    import paper_2601_16991_amd as salr
    M, K, N, R = 4096, 28672, 8192, 64     # even the adapter intermediates alone are beyond the fixed array
    assert salr.salr_linear_workspace_bytes_min(M, K, N, R) > salr.NOALLOC_SCRATCH_BYTES
    fake = 0x1000                          # never dereferenced: the call fails validation first
    st = salr.lib().salr_sparse_lowrank_linear_noalloc(fake, M, K, N, fake, fake, fake, fake, fake, R, fake, None)
    assert st == salr.SALR_ERR_CAPACITY
