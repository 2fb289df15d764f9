"""Pins of the oracle's NF4 quantiser for the packed values (QSALR: paper Sec. 4, "Coupled with Quantization"; the
data type is the 4-bit NormalFloat of the QLoRA paper that the SALR paper cites).  None of these re-types the oracle's
arithmetic: the nearest-entry rule is checked in exact rational arithmetic, the code book against the quantile rule it
is built from, the rest are hand-worked blocks, an error bound and invariants."""
from fractions import Fraction
from statistics import NormalDist

import numpy as np

import oracle
import salr_workloads as wl


def _f32(bits):
    return wl.bf16_bits_to_f32(np.asarray(bits, dtype=np.uint16))


def _unpack(codes, n):
    c = np.empty(2 * codes.size, dtype=np.uint8)
    c[0::2] = codes & 15
    c[1::2] = codes >> 4
    return c[:n]


def test_codebook_is_the_normal_float_code():
    """Ascending, ends at -1 and +1, an exact zero at index 7 (seven negative and eight positive levels), and the
    levels are normal quantiles scaled to [-1, 1]: the positive side is Phi^-1 at nine evenly spaced probabilities
    from 1/2 up to an offset p just below 1, divided by Phi^-1(p); the negative side the same with eight.  The one
    free parameter p is fixed from the level next to +1; every other level must then follow within 0.005."""
    c = oracle.nf4_codebook().astype(np.float64)
    assert c.shape == (16,) and np.all(np.diff(c) > 0)
    assert c[0] == -1.0 and c[15] == 1.0 and c[7] == 0.0
    nd = NormalDist()
    lo, hi = 0.9, 0.9999
    for _ in range(80):
        p = 0.5 * (lo + hi)
        lvl = nd.inv_cdf(0.5 + 7 / 8 * (p - 0.5)) / nd.inv_cdf(p)
        lo, hi = (lo, p) if lvl < c[14] else (p, hi)   # the level falls as p rises (the divisor grows faster)
    p = 0.5 * (lo + hi)
    assert 0.95 < p < 0.99
    pos = [nd.inv_cdf(0.5 + i / 8 * (p - 0.5)) / nd.inv_cdf(p) for i in range(9)]
    assert np.allclose(c[7:], pos, atol=5e-3), (c[7:], pos)
    neg = [-nd.inv_cdf(0.5 + i / 7 * (p - 0.5)) / nd.inv_cdf(p) for i in range(8)]
    assert np.allclose(c[:8][::-1], neg, atol=5e-3), (c[:8][::-1], neg)


def test_hand_worked_blocks():
    """Block 0 has scale 2, the short block 1 scale 8.  By hand, x / scale against the levels:
    -2 -> -1 (code 0); 2 -> +1 (15); 1 -> 0.5: 0.4407 (12) is nearer than 0.5626 (13); -1 -> -0.5: -0.5251 (2);
    0.125 -> 0.0625: 0.0796 (8); 0.25 -> 0.125: 0.1609 (9) is nearer than 0.0796 (8);
    8 -> 1 (15); -4 -> -0.5 (2); 0.5 -> 0.0625 (8)."""
    vals = wl.f32_to_bf16_bits(np.array([-2.0, 2.0, 1.0, -1.0, 0.125] + [0.25] * 59 + [8.0, -4.0, 0.5], dtype=np.float32))
    codes, scales = oracle.nf4_quantize(vals)
    assert codes.size == (67 + 1) // 2 and scales.size == 2
    assert _f32(scales).tolist() == [2.0, 8.0]
    c = _unpack(codes, vals.size)
    assert c[:5].tolist() == [0, 15, 12, 2, 8]
    assert set(c[5:64].tolist()) == {9}
    assert c[64:].tolist() == [15, 2, 8]
    # nibble order: value 0 (code 0) in the low nibble of byte 0, value 1 (code 15) in its high nibble
    assert codes[0] == 0xF0 and codes[1] == (2 << 4 | 12)
    back = _f32(oracle.nf4_dequantize(codes, scales, vals.size))
    lv = oracle.nf4_codebook()
    # dequantised values are level * scale rounded to bf16: -2, 2, 2 * 0.4407..., exact where the level is +-1 or 0
    assert back[0] == -2.0 and back[1] == 2.0 and back[64] == 8.0
    assert abs(back[2] - 2 * lv[12]) <= 2.0 ** -8 * abs(2 * lv[12])


def test_codes_are_the_nearest_level_in_exact_arithmetic():
    """For random bf16 values the code chosen is the level nearest to x / scale, judged with exact rationals on
    x - level * scale (no division, no rounding); where the oracle's fp32 boundary product rounds, the two candidates are
    within one part in 2^23 of equidistant, which the check allows."""
    rng = np.random.default_rng(7)
    vals = wl.gaussian_bf16((64 * 40 + 17,), 0.02, 12345)
    vals[vals == 0] = 0x3C00
    vals[rng.integers(0, vals.size, 50)] = wl.f32_to_bf16_bits(np.float32([0.3]))[0]   # some large entries
    codes, scales = oracle.nf4_quantize(vals)
    c = _unpack(codes, vals.size)
    lv = [Fraction(float(v)) for v in oracle.nf4_codebook()]
    x = _f32(vals)
    s = _f32(scales)
    # every scale is the largest magnitude of its block
    for b in range(scales.size):
        assert s[b] == np.max(np.abs(x[64 * b:64 * b + 64]))
    for i in range(0, vals.size, 7):
        sx, ss = Fraction(float(x[i])), Fraction(float(s[i // 64]))
        dist = [abs(sx - l * ss) for l in lv]
        best = min(dist)
        assert dist[c[i]] <= best + ss * Fraction(1, 2 ** 22), (i, c[i], dist.index(best))


def test_error_bound_idempotence_and_scale_invariance():
    vals = wl.gaussian_bf16((64 * 300,), 0.02, 99)
    vals[(vals & 0x7FFF) == 0] = 0x3C00
    codes, scales = oracle.nf4_quantize(vals)
    back = oracle.nf4_dequantize(codes, scales, vals.size)
    x, xb, s = _f32(vals), _f32(back), np.repeat(_f32(scales), 64)
    lv = oracle.nf4_codebook().astype(np.float64)
    half_gap = 0.5 * np.max(np.diff(lv))                      # the widest gap is at the negative end: (1 - 0.6962) / 2
    assert 0.151 < half_gap < 0.153
    assert np.all(np.abs(x - xb) <= s * half_gap + 2.0 ** -8 * s)
    # the entry that sets the scale is reproduced exactly (level -1 or +1 times the scale)
    for b in range(0, scales.size, 13):
        blk = slice(64 * b, 64 * b + 64)
        j = int(np.argmax(np.abs(x[blk])))
        assert xb[blk][j] == x[blk][j]
    # quantising the dequantised values gives the same codes and scales (levels and scale are fixed points) wherever the
    # block still holds a +-1 level, i.e. always
    codes2, scales2 = oracle.nf4_quantize(back)
    assert np.array_equal(scales2, scales) and np.array_equal(codes2, codes)
    # doubling every value (exact in bf16) doubles the scales and leaves the codes alone
    doubled = (vals + 0x0080).astype(np.uint16)               # exponent + 1
    codes3, scales3 = oracle.nf4_quantize(doubled)
    assert np.array_equal(codes3, codes) and np.array_equal(_f32(scales3), 2 * _f32(scales))


def test_zero_block_and_empty_input():
    codes, scales = oracle.nf4_quantize(np.zeros(5, dtype=np.uint16))
    assert scales.tolist() == [0] and _unpack(codes, 5).tolist() == [7] * 5
    assert oracle.nf4_dequantize(codes, scales, 5).tolist() == [0] * 5
    codes, scales = oracle.nf4_quantize(np.zeros(0, dtype=np.uint16))
    assert codes.size == 0 and scales.size == 0
    # a negative zero in a block counts as magnitude 0 and takes the zero level
    codes, scales = oracle.nf4_quantize(np.array([0x8000, 0x3F80], dtype=np.uint16))
    assert _unpack(codes, 2).tolist() == [7, 15]
