"""Pins for the oracle of the integer path (int8 activations x int4 weights with integer scales; the paper's
closing section, last paragraph, read as stated in oracle/fq_oracle_int.py).

Everything is re-derived here with exact rationals and an independently written correctly rounded binary32
division; the remaining checks are invariants and special cases that reduce to the floating-point format.
A dropped factor (the 16, the 15, the 2), a scale rounded down or to nearest, truncation instead of rounding,
a transposed operand or a z applied to the wrong group fails at least one of them.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads


def _fr(x) -> Fraction:
    return Fraction(float(x))


def _round_half_even(x: Fraction) -> int:
    fl = x.numerator // x.denominator
    rem = x - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def _fl32(x: Fraction) -> Fraction:
    """x rounded to the nearest binary32 value, ties to even (normal and subnormal range, no overflow)."""
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    x = abs(x)
    e = 0
    while Fraction(2) ** e > x:
        e -= 1
    while Fraction(2) ** (e + 1) <= x:
        e += 1
    e = max(e, -126)
    ulp = Fraction(2) ** (e - 23)
    return sign * _round_half_even(x / ulp) * ulp


def _prev_f16(t: np.float16) -> np.float16:
    return np.nextafter(t, np.float16(-np.inf))


def _special_weights():
    """Columns with ties, a zero group, a zero column, subnormals, the largest finite values, groups of very
    different widths (z = 1 next to z = 16)."""
    K, N, g = 128, 8, 32
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((K, N)) * 0.05).astype(np.float16)
    W[:32, 0] = 0                                   # zero group
    W[:, 1] = 0                                     # zero column
    W[:32, 2] = np.float16(6e-8)                    # subnormals only in this group
    W[32:, 2] *= np.float16(1e-3)
    W[5, 3] = np.float16(65504.0)
    W[40, 3] = np.float16(-65504.0)
    W[64:96, 4] = (W[64:96, 4].astype(np.float32) * 1e-3).astype(np.float16)   # a group 1000 times narrower
    W[:, 5] = np.float16(0.75)                      # constant magnitude: every group equally wide
    W[::2, 5] *= np.float16(-1)
    # exact ties: s = z * t with t = 2^-6 (max 3.75 = 240 * 2^-6 / ... see below), weights at (k + 1/2) * s
    W[:, 6] = 0
    W[0, 6] = np.float16(3.75)                      # column max 3.75: 2 * 3.75 / 240 = 2^-5 = t exactly
    W[32:64, 6] = 0
    W[32, 6] = np.float16(0.46875)                  # group max 0.46875: 15 z 2^-5 >= 0.9375 -> z = 2, s = 2^-4
    W[33, 6] = np.float16(1.5 * 2 ** -4)            # quotient 1.5 -> 2 (ties to even)
    W[34, 6] = np.float16(2.5 * 2 ** -4)            # quotient 2.5 -> 2
    W[35, 6] = np.float16(-0.5 * 2 ** -4)           # quotient -0.5 -> 0
    return W, g


def _check_weights_exact(W, g):
    q, z, t = oracle.quantize_int_scales(W, g)
    K, N = W.shape
    assert q.dtype == np.int8 and z.dtype == np.uint8 and t.dtype == np.float16
    assert z.shape == (K // g, N) and t.shape == (N,)
    for n in range(N):
        mcol = max(abs(_fr(w)) for w in W[:, n])
        tn = _fr(t[n])
        assert 240 * tn >= 2 * mcol                                   # covers the widest group
        if tn > 0:
            assert 240 * _fr(_prev_f16(t[n])) < 2 * mcol              # and no smaller binary16 value does
        else:
            assert mcol == 0
        for i in range(K // g):
            grp = W[i * g:(i + 1) * g, n]
            m = max(abs(_fr(w)) for w in grp)
            zi = int(z[i, n])
            assert 1 <= zi <= 16
            if tn == 0:
                assert zi == 1 and not q[i * g:(i + 1) * g, n].any()
                continue
            assert 15 * zi * tn >= 2 * m                              # the group's range is covered
            assert zi == 1 or 15 * (zi - 1) * tn < 2 * m              # by the smallest multiplier
            s = zi * tn
            for k in range(g):
                w = _fr(grp[k])
                want = max(-7, min(7, _round_half_even(_fl32(w / s))))
                assert int(q[i * g + k, n]) == want, (n, i, k)
                assert abs(want * s - w) <= s / 2                     # Appendix A's bound, exactly
                assert abs(want * zi) <= 112


def test_weights_special_values_exact():
    W, g = _special_weights()
    _check_weights_exact(W, g)
    q, z, t = oracle.quantize_int_scales(W, g)
    assert z[0, 1] == 1 and t[1] == 0                                 # zero column
    assert not q[:32, 0].any()                                        # zero group: all codes zero
    assert float(t[6]) == 2.0 ** -5 and z[1, 6] == 2
    assert [int(v) for v in q[33:36, 6]] == [2, 2, 0]                 # the three ties, to even
    assert z[2, 4] == 1 and z[0, 4] > 8                               # a narrow group takes the coarse step
    assert np.all(z[:, 5] == 16)                                      # equally wide groups


@pytest.mark.parametrize("g", [32, 64])
def test_weights_random_exact(g):
    W = workloads.weights_gaussian(128, 6, seed=31 + g, outlier_prob=2e-2)
    _check_weights_exact(W, g)


def test_reduces_to_the_floating_point_format_when_groups_are_equally_wide():
    """Every group of a column with the same abs-max: z = 16 everywhere, 16 t is Appendix A's half-precision
    scale of the group and the codes are those of the floating-point format."""
    rng = np.random.default_rng(9)
    K, N, g = 256, 16, 64
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float16)
    top = np.float16(0.11)
    for i in range(K // g):
        blk = W[i * g:(i + 1) * g]
        np.clip(blk, -top, top, out=blk)
        blk[rng.integers(0, g), :] = top
    q, z, t = oracle.quantize_int_scales(W, g)
    q_f, s_f = oracle.quantize(W, 4, g)
    assert np.all(z == 16)
    assert np.array_equal((t.astype(np.float32) * 16).astype(np.float16)[None, :].repeat(K // g, 0), s_f)
    assert np.array_equal(q, q_f)


def test_bound_and_ranges_on_a_layer_sized_sample():
    W = workloads.opt175b_weight("out_proj", seed=2, rows=1024, cols=512)
    for g in (32, 128, 0):
        q, z, t = oracle.quantize_int_scales(W, g)
        assert q.min() >= -7 and q.max() <= 7 and z.min() >= 1 and z.max() <= 16
        gg = g or W.shape[0]
        s = np.repeat(z.astype(np.float64), gg, axis=0) * t.astype(np.float64)[None, :]
        err = np.abs(oracle.dequantize_int_scales(q, z, t) - W.astype(np.float64))     # exact in float64
        assert np.all(err <= s / 2)
        assert np.all(np.abs(q.astype(np.int32) * np.repeat(z.astype(np.int32), gg, axis=0)) <= 112)
        # the widest group of every column takes the largest multiplier
        assert np.all(z.max(axis=0)[t > 0] == 16)
        # sign symmetry and power-of-two equivariance of the encoder
        q2, z2, t2 = oracle.quantize_int_scales((-W).astype(np.float16), g)
        assert np.array_equal(q2, -q) and np.array_equal(z2, z) and np.array_equal(t2, t)
        q3, z3, t3 = oracle.quantize_int_scales((W.astype(np.float32) * 4).astype(np.float16), g)
        assert np.array_equal(q3, q) and np.array_equal(z3, z) and np.array_equal(t3.astype(np.float32), t.astype(np.float32) * 4)


def test_activations_exact():
    rng = np.random.default_rng(3)
    A = (rng.standard_normal((6, 96)) * 1.3).astype(np.float16)
    A[1] = 0                                                          # zero row
    A[2, 7] = np.float16(-65504.0)
    A[3] = (A[3].astype(np.float32) * 1e-4).astype(np.float16)        # tiny row, subnormals included
    A[4, :] = np.float16(0.5)
    A[4, 3] = np.float16(63.75)                                       # alpha = 0.5 exactly: quotients 1.0 and 127.5
    a, alpha = oracle.quantize_activations_int8(A)
    assert a.dtype == np.int8 and alpha.dtype == np.float32
    for m in range(A.shape[0]):
        amax = max(abs(_fr(v)) for v in A[m])
        al = _fr(alpha[m])
        assert 255 * al >= 2 * amax
        if al > 0:
            assert 255 * _fr(np.nextafter(alpha[m], np.float32(-np.inf))) < 2 * amax
        else:
            assert amax == 0 and not a[m].any()
            continue
        for k in range(A.shape[1]):
            v = _fr(A[m, k])
            want = max(-127, min(127, _round_half_even(_fl32(v / al))))
            assert int(a[m, k]) == want
            assert abs(want * al - v) <= al * (Fraction(1, 2) + Fraction(1, 2 ** 16))
        assert max(abs(int(v)) for v in a[m]) == 127                  # the row's extreme element
    assert float(alpha[4]) == 0.5 and int(a[4, 3]) == 127 and int(a[4, 0]) == 1
    # bfloat16 activations (held in float32) go through the same arithmetic
    B = workloads.activations(3, 64, "bf16", 4)
    b, beta = oracle.quantize_activations_int8(B)
    for m in range(3):
        al = _fr(beta[m])
        for k in range(64):
            assert int(b[m, k]) == max(-127, min(127, _round_half_even(_fl32(_fr(B[m, k]) / al))))


def test_integer_product_brute_force_and_special_cases():
    rng = np.random.default_rng(12)
    M, K, N, g = 3, 64, 5, 32
    a = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    q = rng.integers(-7, 8, size=(K, N)).astype(np.int8)
    z = rng.integers(1, 17, size=(K // g, N)).astype(np.uint8)
    t = (rng.random(N) * 0.01).astype(np.float16)
    alpha = (rng.random(M) * 0.05).astype(np.float32)
    S, C = oracle.gemm_ref_int(a, alpha, q, z, t)
    for m in range(M):
        for n in range(N):
            acc = 0
            for k in range(K):
                acc += int(a[m, k]) * int(q[k, n]) * int(z[k // g, n])
            assert int(S[m, n]) == acc
            assert C[m, n] == pytest.approx(float(_fr(alpha[m]) * _fr(t[n]) * acc), rel=1e-15)
    # one-hot row: S is 127 times one row of q * z
    a1 = np.zeros((1, K), dtype=np.int8)
    a1[0, 37] = 127
    S1, _ = oracle.gemm_ref_int(a1, alpha[:1], q, z, t)
    assert np.array_equal(S1[0], 127 * q[37].astype(np.int64) * z[37 // g].astype(np.int64))
    # additivity in the activations and the largest possible sum
    S2, _ = oracle.gemm_ref_int((a // 2).astype(np.int8), alpha, q, z, t)
    S3, _ = oracle.gemm_ref_int((a - a // 2).astype(np.int8), alpha, q, z, t)
    assert np.array_equal(S2 + S3, S)
    assert 131072 * 127 * 112 < 2 ** 31
    Kb = 4096
    Sb, _ = oracle.gemm_ref_int(np.full((1, Kb), 127, np.int8), alpha[:1], np.full((Kb, 1), -7, np.int8),
                                np.full((Kb // g, 1), 16, np.uint8), t[:1])
    assert int(Sb[0, 0]) == -Kb * 127 * 112


def test_whole_chain_stays_within_the_quantisation_error_bounds():
    """|C - A W| <= sum_k ( |A_k| s_k / 2 + |q z t|_k alpha (1/2 + 2^-16) ): both quantisers' bounds chained."""
    W = workloads.opt175b_weight("qkv", seed=1, rows=512, cols=96)
    A = workloads.activations(7, 512, "f16", 19)
    for g in (64, 128):
        q, z, t = oracle.quantize_int_scales(W, g)
        a, alpha = oracle.quantize_activations_int8(A)
        _, C = oracle.gemm_ref_int(a, alpha, q, z, t)
        A64, W64 = A.astype(np.float64), W.astype(np.float64)
        s = np.repeat(z.astype(np.float64), g, axis=0) * t.astype(np.float64)[None, :]
        What = oracle.dequantize_int_scales(q, z, t)
        bound = np.abs(A64) @ (s / 2) + (alpha.astype(np.float64)[:, None] * (0.5 + 2.0 ** -16)) * np.abs(What).sum(axis=0)[None, :]
        assert np.all(np.abs(C - A64 @ W64) <= bound * (1 + 1e-12))
    # without outliers the groups of a column are about equally wide, the multipliers stay near 16 and the result
    # is close to the weight-only (fp16-activation) one
    Wg = workloads.weights_gaussian(512, 96, seed=23)
    q, z, t = oracle.quantize_int_scales(Wg, 128)
    assert z.min() >= 8
    _, C = oracle.gemm_ref_int(a, alpha, q, z, t)
    qf, sf = oracle.quantize(Wg, 4, 128)
    Cf = oracle.gemm_ref(A, qf, sf)
    assert np.max(np.abs(C - Cf)) <= 0.1 * np.max(np.abs(Cf))
