"""Pins for the oracle's product (section 4.1, "GPU kernel implementations") and for the
adaptive group-size heuristic (section 3.3)."""
import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads


def _case(M, K, N, bits, g, seed, dtype="f16"):
    A = workloads.activations(M, K, dtype, seed)
    W = workloads.weights_gaussian(K, N, seed + 1, outlier_prob=0.01)
    q, s = oracle.quantize(W, bits, g)
    return A, W, q, s


# ------------------------------------------------------------------ product
@pytest.mark.parametrize("bits,g", [(4, 8), (8, 0), (4, 16)])
def test_gemm_matches_brute_force_triple_loop(bits, g):
    A, W, q, s = _case(3, 32, 5, bits, g, seed=5)
    C = oracle.gemm_ref(A, q, s, col_block=2)             # odd block to cross block borders
    gg = g or 32
    for m in range(3):
        for n in range(5):
            acc = 0.0
            for k in range(32):
                acc += float(A[m, k]) * (int(q[k, n]) * float(s[k // gg, n]))
            assert abs(acc - C[m, n]) <= 1e-12 * max(1.0, abs(acc))


def test_gemm_one_hot_row_reads_back_dequantised_weights():
    """A = e_k picks row k of the dequantised matrix: catches a transposed operand or a wrong group index."""
    _, W, q, s = _case(1, 64, 24, 4, 16, seed=9)
    for k in (0, 15, 16, 47, 63):
        A = np.zeros((1, 64), dtype=np.float16)
        A[0, k] = 1.0
        C = oracle.gemm_ref(A, q, s)
        expect = q[k].astype(np.float64) * s[k // 16].astype(np.float64)
        assert np.array_equal(C[0], expect)
        # and that row is within half a step of the original weights
        assert np.all(np.abs(C[0] - W[k].astype(np.float64)) <= s[k // 16].astype(np.float64) / 2)


def test_gemm_all_ones_codes_give_row_sums_and_is_linear():
    K, N, M = 48, 7, 4
    q = np.ones((K, N), dtype=np.int8)
    s = np.ones((K // 16, N), dtype=np.float16)
    A = workloads.activations(M, K, "f16", 3)
    C = oracle.gemm_ref(A, q, s)
    rs = A.astype(np.float64).sum(axis=1)
    assert np.allclose(C, np.repeat(rs[:, None], N, axis=1), rtol=0, atol=1e-12)
    # linearity in A, and scaling one group's scale scales only that group's contribution
    A2 = workloads.activations(M, K, "f16", 4)
    _, _, q2, s2 = _case(M, K, N, 4, 16, seed=13)
    lhs = oracle.gemm_ref(A.astype(np.float64) + 2.0 * A2.astype(np.float64), q2, s2)
    rhs = oracle.gemm_ref(A, q2, s2) + 2.0 * oracle.gemm_ref(A2, q2, s2)
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    s3 = s2.copy()
    s3[1] = (s3[1].astype(np.float32) * 2).astype(np.float16)
    diff = oracle.gemm_ref(A, q2, s3) - oracle.gemm_ref(A, q2, s2)
    part = A.astype(np.float64)[:, 16:32] @ (q2[16:32].astype(np.float64) * s2[1].astype(np.float64))
    assert np.allclose(diff, part, rtol=1e-10, atol=1e-12)


def test_gemm_close_to_unquantised_product():
    """The quantised product approximates A.W with an error governed by s/2 per weight."""
    A, W, q, s = _case(4, 256, 32, 8, 64, seed=17)
    C = oracle.gemm_ref(A, q, s)
    C0 = A.astype(np.float64) @ W.astype(np.float64)
    bound = np.abs(A.astype(np.float64)) @ np.repeat(s.astype(np.float64) / 2, 64, axis=0)
    assert np.all(np.abs(C - C0) <= bound + 1e-12)
    assert np.max(np.abs(C - C0)) > 0


def test_gemm_bf16_activations_are_taken_exactly():
    A = workloads.activations(2, 64, "bf16", 23)
    assert np.array_equal(workloads.bf16_from_bits(workloads.bf16_bits(A)), A)
    _, _, q, s = _case(2, 64, 8, 4, 32, seed=29)
    C = oracle.gemm_ref(A, q, s)
    assert C.dtype == np.float64
    assert np.allclose(C, A.astype(np.float64) @ oracle.dequantize(q, s), rtol=0, atol=0)


def test_grouped_product_skips_empty_experts():
    E, K, N = 4, 32, 8
    rows = [3, 0, 5, 1]
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    A = workloads.activations(int(offsets[-1]), K, "f16", 31)
    qs, ss = [], []
    for e in range(E):
        W = workloads.weights_gaussian(K, N, 40 + e)
        q, s = oracle.quantize(W, 4, 16)
        qs.append(q)
        ss.append(s)
    C = oracle.gemm_ref_grouped(A, offsets, qs, ss)
    for e in range(E):
        r0, r1 = offsets[e], offsets[e + 1]
        for r in range(r0, r1):
            expect = A[r].astype(np.float64) @ oracle.dequantize(qs[e], ss[e])
            assert np.allclose(C[r], expect, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- heuristic
def test_constant_magnitude_matrix_keeps_the_start_size():
    W = np.full((256, 16), 0.5, dtype=np.float16)
    W[::3] *= -1
    assert oracle.choose_group(W, 0, 32, 0.5) == 256
    assert oracle.choose_group(W, 128, 32, 0.01) == 128


def _planted(K, N, level_size, k_pos, big=8.0, base=1.0):
    """|w| = base everywhere, except one element of magnitude ``big`` at row k_pos of column 0."""
    W = np.full((K, N), base, dtype=np.float16)
    W[k_pos, 0] = np.float16(big)
    return W


def test_single_outlier_drives_halving_all_the_way_down():
    # at every level the outlier's sibling half has range 1 = parent/8 -> relative difference 0.875
    W = _planted(512, 4, None, 5)
    assert oracle.choose_group(W, 0, 32, 0.5) == 32
    assert oracle.choose_group(W, 0, 128, 0.5) == 128          # g_min stops it
    assert oracle.choose_group(W, 0, 32, 0.9) == 512           # 0.875 is not more than 0.9
    assert oracle.choose_group(W, 256, 64, 0.5) == 64


def test_structure_visible_only_down_to_one_level():
    """A block of large rows is seen only down to the level where both halves of every parent agree.

    Column 0 has magnitude 8 at rows 0..63 and 1 elsewhere (K = 512).
    512 -> 256: children (8, 1)  -> halve.   256 -> 128: (8, 1) -> halve.
    128 -> 64: in the first parent children are (8, 1) -> halve.
    64 -> 32: every parent has equal children (8, 8) or (1, 1) -> stop at 64.
    """
    W = np.full((512, 3), 1.0, dtype=np.float16)
    W[:64, 0] = 8.0
    assert oracle.choose_group(W, 0, 16, 0.5) == 64
    # With 96 large rows the 128 -> 64 test sees equal children (8, 8) in parent [0,128) and (1, 1)
    # elsewhere, so the loop stops at 128 although the 64 -> 32 level would differ again: the
    # procedure ends at the first level whose ranges stop changing.
    W2 = np.full((512, 3), 1.0, dtype=np.float16)
    W2[:96, 0] = 8.0
    assert oracle.choose_group(W2, 0, 16, 0.5) == 128
    assert oracle.choose_group(W2, 64, 16, 0.5) == 32          # started below that level it does see it


def test_threshold_is_strict_and_evaluated_on_relative_difference():
    # children ranges (4, 1): min/parent = 0.25, relative difference 0.75
    W = np.full((64, 2), 1.0, dtype=np.float16)
    W[:32, 1] = 4.0
    assert oracle.choose_group(W, 0, 32, 0.5) == 32            # 0.75 > 0.5 -> halve
    assert oracle.choose_group(W, 0, 32, 0.75) == 64           # 0.75 is not > 0.75 -> stop
    assert oracle.choose_group(W, 0, 32, 0.8) == 64
    # sign does not matter: the range is an abs-max
    W[:32, 1] = -4.0
    assert oracle.choose_group(W, 0, 32, 0.5) == 32


def test_any_group_anywhere_triggers_the_halving():
    rng = np.random.default_rng(0)
    for _ in range(5):
        W = np.full((128, 8), 1.0, dtype=np.float16)
        k = int(rng.integers(0, 128))
        n = int(rng.integers(0, 8))
        W[k, n] = 16.0
        assert oracle.choose_group(W, 0, 64, 0.5) == 64
    W = np.full((128, 8), 1.0, dtype=np.float16)
    assert oracle.choose_group(W, 0, 64, 0.5) == 128


def test_monotone_in_alpha_on_random_weights():
    W = workloads.weights_gaussian(1024, 64, 77, outlier_prob=1e-3)
    prev = 0
    for alpha in (0.1, 0.3, 0.5, 0.7, 0.9, 0.97, 0.995):
        g = oracle.choose_group(W, 256, 32, alpha)
        assert g >= prev
        assert g in (32, 64, 128, 256)
        prev = g
    assert oracle.choose_group(W, 256, 32, 0.0) == 32          # any difference at all triggers halving
    assert oracle.choose_group(W, 256, 32, 1.0) == 256         # nothing is below 0 * parent


def test_odd_factor_stops_halving():
    W = workloads.weights_gaussian(96, 4, 5)                    # 96 -> 48 -> 24 -> 12 -> 6 -> 3
    assert oracle.choose_group(W, 0, 1, 0.0) == 3
    assert oracle.choose_group(W, 0, 32, 0.0) == 48
