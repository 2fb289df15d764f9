"""Pins for the oracle's magnitude mask (paper Sec. 2 and Theorem 1).  CPU only."""
import os

import numpy as np
import pytest

import oracle
import salr_workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "thm1_worked_example.txt")


def _brute_force_mask(row_bits, keep):
    """O(K^2) rank count: an entry is kept iff fewer than `keep` entries beat it, where j beats i when
    |w_j| > |w_i|, or |w_j| == |w_i| and j < i."""
    K = len(row_bits)
    out = [0] * K
    mags = [int(b) & 0x7FFF for b in row_bits]
    for i in range(K):
        beaten_by = 0
        for j in range(K):
            if mags[j] > mags[i] or (mags[j] == mags[i] and j < i):
                beaten_by += 1
        if beaten_by < keep:
            out[i] = int(row_bits[i])
    return out


def test_mask_matches_brute_force_rank_count_with_ties():
    rng = np.random.default_rng(7)
    # few distinct magnitudes => many ties, both signs
    vals = wl.f32_to_bf16_bits(np.array([0.5, -0.5, 0.25, -0.25, 1.0, -1.0, 0.125, 2.0], dtype=np.float32))
    for K, keep in [(8, 4), (13, 5), (32, 16), (40, 0), (40, 40), (33, 1)]:
        w = vals[rng.integers(0, len(vals), size=(6, K))]
        got = oracle.mask_topk_rows(w, keep)
        for n in range(w.shape[0]):
            assert got[n].tolist() == _brute_force_mask(w[n], keep), (K, keep, n)


def test_mask_hand_made_row():
    # magnitudes: 3 1 3 2 2 1 ; keep 3 -> both 3s, then the first of the 2s (lower column)
    row = wl.f32_to_bf16_bits(np.array([[3.0, -1.0, -3.0, 2.0, -2.0, 1.0]], dtype=np.float32))
    got = oracle.mask_topk_rows(row, 3)
    assert got[0].tolist() == [row[0, 0], 0, row[0, 2], row[0, 3], 0, 0]


def test_mask_counts_and_dominance_gaussian():
    cfg = wl.CONFIGS["tiny"]
    w = wl.dense_weight(cfg)
    for permille in (500, 700, 0, 1000):
        keep = cfg.keep(permille)
        w_hat = oracle.mask_topk_rows(w, keep)
        nz = (w_hat & 0x7FFF) != 0
        # generated weights contain no exact zeros among the kept ones
        assert (nz.sum(axis=1) == keep).all()
        assert nz.sum() == cfg.N * keep
        # kept entries are untouched, pruned are +0.0
        assert (w_hat[nz] == w[nz]).all()
        assert (w_hat[~nz] == 0).all()
        mag = (w & 0x7FFF).astype(np.int64)
        if 0 < keep < cfg.K:
            min_kept = np.where(nz, mag, 1 << 20).min(axis=1)
            max_pruned = np.where(~nz, mag, -1).max(axis=1)
            assert (min_kept >= max_pruned).all()


def test_mask_equals_printed_threshold_rule_when_no_ties():
    """Sec. 2 prints: keep iff |w| > T_p.  On a row whose (keep+1)-th magnitude is not tied with the
    keep-th, the per-row top-k mask is that rule with T = the (keep+1)-th largest magnitude."""
    cfg = wl.CONFIGS["tiny"]
    w = wl.dense_weight(cfg, rows=64)
    keep = cfg.keep(500)
    w_hat = oracle.mask_topk_rows(w, keep)
    checked = 0
    for n in range(w.shape[0]):
        mags = np.sort((w[n] & 0x7FFF).astype(np.int64))[::-1]
        t = mags[keep]
        strict = oracle.mask_threshold(w[n:n + 1], int(t))
        if mags[keep - 1] != t:
            assert (strict == w_hat[n:n + 1]).all()
            checked += 1
        else:
            # ties at the threshold: the printed rule keeps a strict subset (it over-prunes)
            kept_strict = (strict & 0x7FFF) != 0
            kept_topk = (w_hat[n:n + 1] & 0x7FFF) != 0
            assert (kept_strict & ~kept_topk).sum() == 0
            assert kept_strict.sum() < keep
    assert checked > 10


def _golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


def test_theorem1_closed_form_against_papers_worked_example():
    g = _golden()
    from statistics import NormalDist
    import math
    t = NormalDist().inv_cdf((1 + g["p"]) / 2)
    assert abs(t - g["t_p"]) < 5e-4
    assert abs(math.exp(-t * t / 2) / math.sqrt(2 * math.pi) - g["phi_t_p"]) < 5e-4
    # the printed threshold, put through the normal CDF, gives the printed (1 + p) / 2
    assert abs(NormalDist().cdf(g["t_p"]) - g["Phi_t_p"]) < 5e-4
    assert abs((1 + g["p"]) / 2 - g["Phi_t_p"]) < 1e-12
    # the paper's 0.072 comes from rounded intermediates (0.25 - 0.214); the exact value is 0.07133
    assert abs(oracle.pruning_mse_closed_form(g["p"]) - g["mse_over_sigma2"]) < 1e-3
    # same arithmetic as printed, with the printed roundings
    assert abs(2 * (g["Phi_t_p"] - 0.5 - g["t_p"] * g["phi_t_p"]) - g["mse_over_sigma2"]) < 1e-3


@pytest.mark.parametrize("permille", [500, 700, 300])
def test_mask_mse_matches_theorem1(permille):
    """Empirical ||W - What||_F^2 / (N K sigma^2) on Gaussian weights vs Theorem 1's closed form."""
    cfg = wl.CONFIGS["tiny"]
    w = wl.dense_weight(cfg)
    keep = cfg.keep(permille)
    w_hat = oracle.mask_topk_rows(w, keep)
    mse, _ = oracle.svd_residual_check(w, w_hat, 0)
    expect = oracle.pruning_mse_closed_form(permille / 1000.0, cfg.std_w)
    assert abs(mse / expect - 1.0) < 0.03, (mse, expect)


def test_nm_mask_is_the_row_mask_applied_per_group():
    """An N:M group is a tiny row: mask_nm(w, n, m) == mask_topk_rows on the groups laid out as rows."""
    rng = np.random.default_rng(11)
    vals = wl.f32_to_bf16_bits(np.array([0.5, -0.5, 0.25, 1.0, -1.0, 0.125, 0.0, -0.0], dtype=np.float32))
    for n, m in [(2, 4), (1, 4), (4, 8), (1, 2), (4, 4), (0, 4)]:
        w = vals[rng.integers(0, len(vals), size=(5, 8 * m))]
        got = oracle.mask_nm(w, n, m)
        expect = oracle.mask_topk_rows(np.ascontiguousarray(w.reshape(-1, m)), n).reshape(w.shape)
        assert np.array_equal(got, expect), (n, m)
    w = wl.gaussian_bf16((16, 256), 0.02, 3)
    got = oracle.mask_nm(w, 2, 4)
    nz = ((got & 0x7FFF) != 0).reshape(16, 64, 4)
    assert (nz.sum(axis=2) == 2).all()          # Gaussian draws have no zeros: exactly 2 of every 4 survive
    assert (got[(got & 0x7FFF) != 0] == w[(got & 0x7FFF) != 0]).all()


def test_nm_mask_hand_made_group():
    # magnitudes 1 3 3 2 -> keep both 3s ; 2 2 2 2 -> ties: the two lowest columns
    w = wl.f32_to_bf16_bits(np.array([[1.0, -3.0, 3.0, 2.0, 2.0, -2.0, 2.0, 2.0]], dtype=np.float32))
    got = oracle.mask_nm(w, 2, 4)
    assert got[0].tolist() == [0, w[0, 1], w[0, 2], 0, w[0, 4], w[0, 5], 0, 0]
