"""Pins for the oracle's bfloat16 scale format (section 4.1, "GPU kernel implementations": the kernels
for bfloat16 activations take scales of the activation's data type; Appendix A for the arithmetic).

Scales and codes are re-derived with exact rationals and integer bit manipulation written here,
independently of the oracle; the remaining checks are invariants a wrong rounding direction, a wrong
mantissa width or a scale taken from the other format would break.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads


def _smallest_bf16_at_least(x: Fraction) -> Fraction:
    """Smallest non-negative bfloat16 value (1 + 7 bit significand, binary32's exponent range) >= x."""
    if x == 0:
        return Fraction(0)
    # e = floor(log2 x), found by exact comparisons
    e = 0
    while Fraction(2) ** e > x:
        e -= 1
    while Fraction(2) ** (e + 1) <= x:
        e += 1
    assert e >= -126                      # normal range; the abs-max of a binary16 group never goes below
    ulp = Fraction(2) ** (e - 7)
    n = x / ulp                           # in [128, 256)
    c = -((-n.numerator) // n.denominator)   # ceiling
    return c * ulp                        # c = 256 is the next binade's first value: still a bfloat16


def _round_half_even(x: Fraction) -> int:
    fl = x.numerator // x.denominator
    rem = x - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def _is_bf16(x: Fraction) -> bool:
    if x == 0:
        return True
    f = np.float32(float(x))
    return Fraction(float(f)) == x and (int(f.view(np.uint32)) & 0xFFFF) == 0


@pytest.mark.parametrize("bits", [4, 8])
def test_every_binary16_absmax_gets_the_minimal_bfloat16_scale(bits):
    """All 31744 non-negative finite binary16 abs-max values: bit pattern and two-sided minimality."""
    m = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16)
    s = oracle.scale_from_absmax(m, bits, "bf16")
    assert s.dtype == np.float32
    b = s.view(np.uint32)
    assert not np.any(b & np.uint32(0xFFFF))                 # bfloat16 values
    L = oracle.levels_of(bits)
    m64 = m.astype(np.float64)
    assert np.all(L * s.astype(np.float64) >= 2 * m64)        # exact in binary64
    prev = (b.astype(np.int64) - 0x10000).clip(min=0).astype(np.uint32).view(np.float32)
    pos = m64 > 0
    assert np.all(L * prev[pos].astype(np.float64) < 2 * m64[pos])
    assert s[0] == 0 and np.all(s[1:] > 0)
    # exact rationals on a spread of the values (every 97th, plus the ends)
    idx = list(range(0, len(m), 97)) + [1, 2, len(m) - 1]
    for i in idx:
        want = _smallest_bf16_at_least(2 * Fraction(float(m[i])) / L)
        assert _is_bf16(want)
        assert Fraction(float(s[i])) == want, (i, float(m[i]))
    assert np.array_equal(oracle.bf16_scale_bits(s), (b >> 16).astype(np.uint16))


@pytest.mark.parametrize("bits", [4, 8])
def test_bracket_between_the_two_formats(bits):
    """Both formats round the same real number 2m/L up: s_f16 <= s_bf16 < s_f16 (1 + 2^-7) wherever the
    binary16 scale is a normal number (its own rounding moves it by less than 2^-10 relative)."""
    m = np.arange(0x0400, 0x7C00, 7, dtype=np.uint16).view(np.float16)
    s16 = oracle.scale_from_absmax(m, bits, "f16").astype(np.float64)
    sb = oracle.scale_from_absmax(m, bits, "bf16").astype(np.float64)
    real = 2 * m.astype(np.float64) / oracle.levels_of(bits)
    assert np.all(sb >= real) and np.all(sb < real * (1 + 2.0 ** -7))
    normal = s16 >= 2.0 ** -14
    assert np.all(sb[normal] >= s16[normal] * (1 - 2.0 ** -10))
    assert np.all(sb[normal] < s16[normal] * (1 + 2.0 ** -7))
    # the coarser format moves at least some scales further up
    assert np.mean(sb > s16) > 0.5


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("g", [4, 32])
def test_codes_and_scales_match_exact_rationals(bits, g):
    W = workloads.weights_gaussian(32, 10, 900 + bits + g, sigma=0.02, outlier_prob=0.02)
    W[:g, 1] = np.float16(0.0)                       # an all-zero group
    W[:g, 2] = np.float16(6e-8)                      # the smallest subnormal everywhere
    W[1, 3] = np.float16(65504.0)
    W[2, 3] = np.float16(-65504.0)
    q, s = oracle.quantize(W, bits, g, "bf16")
    L = oracle.levels_of(bits)
    qm = oracle.qmax_of(bits)
    K, N = W.shape
    for n in range(N):
        for gi in range(K // g):
            col = [Fraction(float(W[k, n])) for k in range(gi * g, (gi + 1) * g)]
            sc = _smallest_bf16_at_least(2 * max(abs(c) for c in col) / L)
            assert Fraction(float(s[gi, n])) == sc
            for i, c in enumerate(col):
                code = 0 if sc == 0 else max(-qm, min(qm, _round_half_even(c / sc)))
                assert q[gi * g + i, n] == code


@pytest.mark.parametrize("bits", [4, 8])
def test_binary32_quotient_decides_like_exact_arithmetic(bits):
    """Every bfloat16 scale of one binade (128 of them) against every binary16 numerator whose quotient
    lies in the code range: rne(fl32(w / s)) equals the exact rne(w / s), ties included."""
    qm = oracle.qmax_of(bits)
    s_bits = np.arange(0x3D80, 0x3E00, dtype=np.uint32) << np.uint32(16)      # [2^-4, 2^-3)
    s_vals = s_bits.view(np.float32)
    f16 = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16)
    w_all = f16[(f16 <= np.float16((qm + 1) * 0.125)) & (f16 >= np.float16(2.0 ** -9))]
    a = np.round(w_all.astype(np.float64) * 2.0 ** 24).astype(np.int64)
    b = np.round(s_vals.astype(np.float64) * 2.0 ** 24).astype(np.int64)
    assert np.array_equal(a * 2.0 ** -24, w_all.astype(np.float64))
    assert np.array_equal(b * 2.0 ** -24, s_vals.astype(np.float64))
    A, B = np.meshgrid(a, b, indexing="ij")
    fl = A // B
    rem2 = 2 * (A - fl * B)
    exact = np.where(rem2 > B, fl + 1, np.where(rem2 < B, fl, fl + (fl & 1)))
    assert int((rem2 == B).sum()) > 100
    got = np.rint(w_all.astype(np.float32)[:, None] / s_vals[None, :]).astype(np.int64)
    assert np.array_equal(got, exact)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("g", [32, 128, 0])
def test_half_step_bound_and_code_range(bits, g):
    W = workloads.weights_gaussian(512, 64, 31 * bits + (g or 1), sigma=0.02, outlier_prob=0.01)
    q, s = oracle.quantize(W, bits, g, "bf16")
    qm = oracle.qmax_of(bits)
    gg = g or W.shape[0]
    assert q.min() >= -qm and q.max() <= qm
    s_rows = np.repeat(s.astype(np.float64), gg, axis=0)
    err = np.abs(q.astype(np.float64) * s_rows - W.astype(np.float64))
    assert np.all(err <= s_rows / 2)
    m = np.abs(W).reshape(-1, gg, W.shape[1]).max(axis=1)
    top = np.abs(q).reshape(-1, gg, W.shape[1]).max(axis=1)
    assert np.all(top[m > 0] == qm)
    # the dequantised matrix stays a faithful copy: the error measure is within 2^-7 of the f16 format's
    q16, s16 = oracle.quantize(W, bits, g, "f16")
    e_b = oracle.quant_error(W, q, s)[0]
    e_h = oracle.quant_error(W, q16, s16)[0]
    assert abs(e_b - e_h) <= 0.05 * e_h


def test_power_of_two_equivariance_and_sign_symmetry():
    W = workloads.weights_gaussian(128, 32, 77, sigma=0.02, outlier_prob=0.01)
    for bits in (4, 8):
        q, s = oracle.quantize(W, bits, 32, "bf16")
        q2, s2 = oracle.quantize((W.astype(np.float32) * 16).astype(np.float16), bits, 32, "bf16")
        assert np.array_equal(q, q2) and np.array_equal(s2, s * np.float32(16))
        q3, s3 = oracle.quantize(-W, bits, 32, "bf16")
        assert np.array_equal(q3, -q) and np.array_equal(s3, s)


def test_format_argument_is_checked():
    m = np.ones((1, 1), dtype=np.float16)
    with pytest.raises(ValueError):
        oracle.scale_from_absmax(m, 4, "f32")
    with pytest.raises(ValueError):
        oracle.bf16_scale_bits(np.array([1.0000001], dtype=np.float32))
