"""Pins for the oracle's quantisation-error measure (section 3.2, figure 2a: mean squared error of the
quantise / dequantise round trip; dequantised value per Appendix A).

The reference values come from exact rational arithmetic on an independently written quantiser, from
closed forms and from invariants; none re-types the oracle's floating-point expression.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads

from test_oracle_quantizer import _exact_quantize


def _exact_error(W, bits, g):
    """(sum of squared errors, max abs error) as exact rationals, from the rational quantiser."""
    q, s = _exact_quantize(W, bits, g)
    K, N = W.shape
    sse = Fraction(0)
    mx = Fraction(0)
    for n in range(N):
        for k in range(K):
            e = Fraction(float(W[k, n])) - q[k, n] * Fraction(float(s[k // g, n]))
            sse += e * e
            mx = max(mx, abs(e))
    return sse, mx


@pytest.mark.parametrize("bits,g", [(4, 32), (4, 64), (8, 32), (8, 64)])
def test_matches_exact_rational_round_trip(bits, g):
    W = workloads.weights_gaussian(64, 6, seed=70 + bits + g, outlier_prob=0.02)
    q, s = oracle.quantize(W, bits, g)
    sse, mx = oracle.quant_error(W, q, s)
    sse_x, mx_x = _exact_error(W, bits, g)
    assert mx == float(mx_x)                                   # a single exact difference: bit-exact
    assert abs(sse - float(sse_x)) <= 1e-13 * float(sse_x)     # 384 exact squares summed in fp64


def test_constant_column_has_the_closed_form_error():
    """All weights equal to c: the code is the clamped top code, the error c - qmax * s for every element."""
    for bits in (4, 8):
        qm = (1 << (bits - 1)) - 1
        c = np.float16(0.3701171875)
        W = np.full((64, 3), c, dtype=np.float16)
        W[::2, 1] = -c                                         # signs do not matter
        q, s = oracle.quantize(W, bits, 64)
        assert np.all(np.abs(q) == qm)
        e = Fraction(float(c)) - qm * Fraction(float(s[0, 0]))
        sse, mx = oracle.quant_error(W, q, s)
        assert mx == abs(float(e))
        assert abs(sse - float(W.size * e * e)) <= 1e-14 * float(W.size * e * e)


def test_error_never_exceeds_half_a_step_and_sse_is_bounded_by_it():
    W = workloads.weights_heavy_tail(256, 48, seed=5)
    for bits in (4, 8):
        for g in (32, 128, 256):
            q, s = oracle.quantize(W, bits, g)
            sse, mx = oracle.quant_error(W, q, s)
            smax = float(np.max(s.astype(np.float64)))
            assert mx <= smax / 2
            assert sse <= W.size * (smax / 2) ** 2
            assert sse > 0


def test_uniformly_spread_weights_give_a_twelfth_of_the_squared_step():
    """Weights uniform in [-m, m] leave errors uniform in [-s/2, s/2]: MSE -> s^2 / 12 (here within 3 %)."""
    rng = np.random.default_rng(3)
    K, N = 4096, 8
    W = rng.uniform(-1.0, 1.0, size=(K, N)).astype(np.float16)
    W[0, :] = 1.0                                              # pin the abs-max of every column
    for bits in (4, 8):
        q, s = oracle.quantize(W, bits, K)
        sse, _ = oracle.quant_error(W, q, s)
        step = float(s[0, 0])
        assert abs(step - 2.0 / ((1 << bits) - 1)) < 1e-3 * step
        mse = sse / W.size
        tol = 0.03 if bits == 4 else 0.06                      # fp16 spacing of the inputs shows at 8 bits
        assert abs(mse - step * step / 12.0) <= tol * step * step / 12.0


def test_additive_over_column_blocks_and_equivariant_under_powers_of_two():
    W = workloads.weights_gaussian(128, 32, seed=9, sigma=1.0)
    q, s = oracle.quantize(W, 4, 64)
    sse, mx = oracle.quant_error(W, q, s)
    parts = [oracle.quant_error(W[:, a:a + 8], q[:, a:a + 8], s[:, a:a + 8]) for a in range(0, 32, 8)]
    assert abs(sum(p[0] for p in parts) - sse) <= 1e-13 * sse
    assert max(p[1] for p in parts) == mx
    W4 = (W.astype(np.float32) * 4).astype(np.float16)         # exact scaling (values stay normal, finite)
    q4, s4 = oracle.quantize(W4, 4, 64)
    assert np.array_equal(q4, q)
    sse4, mx4 = oracle.quant_error(W4, q4, s4)
    assert mx4 == 4 * mx
    assert abs(sse4 - 16 * sse) <= 1e-13 * sse4


def test_finer_groups_never_increase_the_largest_error_bound():
    """Child scale <= parent scale, hence the s/2 bound shrinks (section 3.2's motivation for small groups)."""
    W = workloads.weights_gaussian(256, 64, seed=12, outlier_prob=0.01)
    prev = None
    for g in (256, 128, 64, 32):
        q, s = oracle.quantize(W, 4, g)
        sse, mx = oracle.quant_error(W, q, s)
        bound = float(np.max(s.astype(np.float64))) / 2
        assert mx <= bound
        if prev is not None:
            assert bound <= prev
        prev = bound
