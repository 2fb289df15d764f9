"""GPU parity: salr_sparse_lowrank_linear_backward through the C boundary vs the fp64 CPU oracle.

Bar, as for the forward pass: max |G - G_ref| <= 1e-2 * max |G_ref| for each of dX, dA, dB (bf16 inputs, two bf16-rounded
[M, R] intermediates, fp32 sums, bf16 outputs)."""
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


def _close(g, ref, label):
    scale, err = float(np.max(np.abs(ref))), float(np.max(np.abs(g - ref)))
    print(f"[backward] {label}: max|d|={err:.3e} scale={scale:.3e} rel={err / scale:.2e}", flush=True)
    assert err <= REL_TOL * scale, label


def _problem(M, K, N, ranks, seed):
    x = wl.gaussian_bf16((M, K), 1.0, seed)
    dy = wl.gaussian_bf16((M, N), 1.0, seed + 1)
    w_hat = oracle.mask_topk_rows(wl.gaussian_bf16((N, K), 0.02, seed + 2), K // 2)
    if ranks:
        As = [wl.gaussian_bf16((K, r), 0.05, seed + 10 + i) for i, r in enumerate(ranks)]
        Bs = [wl.gaussian_bf16((r, N), 0.05, seed + 20 + i) for i, r in enumerate(ranks)]
        a_cat, b_cat = wl.concat_adapters(As, Bs)
    else:
        a_cat = b_cat = None
    return x, dy, w_hat, a_cat, b_cat


def _run(x, dy, w_hat, a_cat, b_cat, need_dx=True, need_dadb=True):
    salr = _salr()
    rb, rv, ro = oracle.encode(w_hat)
    out = salr.linear_backward(to_dev_u16(x), to_dev_u16(dy), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro),
                               None if a_cat is None else to_dev_u16(a_cat), None if b_cat is None else to_dev_u16(b_cat),
                               need_dx, need_dadb)
    torch.cuda.synchronize()
    return [None if t is None else y_to_f64(t) for t in out]


@pytest.mark.parametrize("M,K,N,ranks", [(32, 64, 64, (8,)), (96, 256, 192, (16, 8)), (256, 512, 320, (40,)),
                                        (64, 1024, 128, (32, 32, 64)), (320, 96, 704, (5, 3)), (2048, 512, 512, (16,)),
                                        # K a multiple of 128: the weight is decoded straight into its transpose; one chunk per
                                        # row, one slice of many chunks, many slices
                                        (128, 384, 128, (8,)), (64, 256, 192, (4,)), (96, 4096, 320, (16,)), (160, 128, 64, (2,)),
                                        (64, 2048, 4160, (8,)),
                                        # adapter gradients: column counts of X / dY that are not whole 64-column blocks or not a
                                        # multiple of 8, ranks of one and of many 16-column tiles, a single 32-row step
                                        (32, 96, 64, (3,)), (96, 160, 192, (16, 16, 16)), (64, 1056, 128, (64, 64, 64, 64)),
                                        (1024, 4096, 4096, (32,))])
def test_backward_all_gradients(M, K, N, ranks):
    x, dy, w_hat, a_cat, b_cat = _problem(M, K, N, ranks, 1000 + M + K + N)
    dx, da, db = _run(x, dy, w_hat, a_cat, b_cat)
    rx, ra, rb_ = oracle.linear_backward(x, dy, w_hat, a_cat, b_cat)
    _close(dx, rx, f"dX M{M} K{K} N{N} R{sum(ranks)}")
    _close(da, ra, f"dA M{M} K{K} N{N} R{sum(ranks)}")
    _close(db, rb_, f"dB M{M} K{K} N{N} R{sum(ranks)}")


@pytest.mark.parametrize("M", [1, 40, 300])
def test_backward_input_gradient_only(M):
    """dX alone needs no multiple-of-32 batch; without adapters it is dY times the decoded weight."""
    x, dy, w_hat, a_cat, b_cat = _problem(M, 256, 128, (8,), 2000 + M)
    dx, da, db = _run(x, dy, w_hat, a_cat, b_cat, need_dadb=False)
    assert da is None and db is None
    _close(dx, oracle.linear_backward(x, dy, w_hat, a_cat, b_cat)[0], f"dX only, M={M}")
    dx0, _, _ = _run(x, dy, w_hat, None, None)
    _close(dx0, oracle.linear_backward(x, dy, w_hat, None, None)[0], f"dX, no adapters, M={M}")


def test_backward_adapter_gradients_only():
    x, dy, w_hat, a_cat, b_cat = _problem(128, 256, 192, (24,), 3000)
    dx, da, db = _run(x, dy, w_hat, a_cat, b_cat, need_dx=False)
    assert dx is None
    _, ra, rb_ = oracle.linear_backward(x, dy, w_hat, a_cat, b_cat)
    _close(da, ra, "dA only")
    _close(db, rb_, "dB only")


def test_backward_is_adjoint_to_the_gpu_forward():
    """<dY, Y> = <dX, X> between the two GPU entry points themselves (bf16 rounding on both sides: 1 %)."""
    salr = _salr()
    x, dy, w_hat, a_cat, b_cat = _problem(64, 512, 256, (16,), 4000)
    rb, rv, ro = oracle.encode(w_hat)
    d = [to_dev_u16(x), to_dev_u32(rb), to_dev_u16(rv), to_dev_u32(ro), to_dev_u16(a_cat), to_dev_u16(b_cat)]
    y = y_to_f64(salr.linear(*d))
    dx = _run(x, dy, w_hat, a_cat, b_cat, need_dadb=False)[0]
    lhs, rhs = np.sum(oracle.bf16_to_f64(dy) * y), np.sum(dx * oracle.bf16_to_f64(x))
    assert abs(lhs - rhs) <= 1e-2 * np.sqrt(np.sum((oracle.bf16_to_f64(dy) * y) ** 2) * y.size) / np.sqrt(y.size)


def test_backward_q_proj_full_size():
    cfg = wl.CONFIGS["llama3_8b_q_proj"]
    M = 512
    x = wl.activations(cfg, M)
    dy = wl.gaussian_bf16((M, cfg.N), 1.0, 77)
    w_hat = oracle.mask_topk_rows(wl.dense_weight(cfg), cfg.keep(500))
    a_cat, b_cat = wl.concat_adapters(*wl.adapters(cfg))
    dx, da, db = _run(x, dy, w_hat, a_cat, b_cat)
    rx, ra, rb_ = oracle.linear_backward(x, dy, w_hat, a_cat, b_cat)
    _close(dx, rx, "q_proj dX")
    _close(da, ra, "q_proj dA")
    _close(db, rb_, "q_proj dB")
