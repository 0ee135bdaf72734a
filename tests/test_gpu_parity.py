"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Codes and scales must match bit for bit; products must satisfy
max|C - C_ref| <= 4e-3 max|C_ref| (fp16) / 1.6e-2 max|C_ref| (bf16).
"""
import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads

from gpu_util import (TOL, assert_gemm_close, assert_quantizer_parity, from_dev_act, gpu_quantize, round_to_act,
                      to_dev_act, torch_mod)

pytestmark = pytest.mark.gpu


def _fq():
    from paper_2308_09723_amd import fq
    return fq


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ quantiser
@pytest.mark.parametrize("bits,g", [(8, 0), (4, 128)])
def test_quantize_config1(bits, g):
    _say(f"quantize config1 bits={bits} g={g}")
    _, W = workloads.config1(0)
    assert_quantizer_parity(W, bits, g)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("K,N,g", [(384, 80, 32), (512, 272, 64), (768, 48, 96), (1024, 16, 0), (256, 1040, 256)])
def test_quantize_ragged_shapes_and_outliers(bits, K, N, g):
    _say(f"quantize ragged bits={bits} K={K} N={N} g={g}")
    W = workloads.weights_gaussian(K, N, seed=K + N + bits, outlier_prob=0.01)
    assert_quantizer_parity(W, bits, g)
    Wh = workloads.weights_heavy_tail(K, N, seed=K + N + bits + 1, col_prob=0.05)
    assert_quantizer_parity(Wh, bits, g)


@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_edge_values(bits):
    _say(f"quantize edge values bits={bits}")
    K, N, g = 256, 32, 64
    W = workloads.weights_gaussian(K, N, seed=99)
    W[:, 0] = 0                                   # all-zero column
    W[:64, 1] = 0                                 # one all-zero group
    W[:, 2] = np.float16(6e-8)                    # smallest subnormal everywhere
    W[64:128, 3] = np.float16(6e-8)
    W[70, 3] = np.float16(-1.2e-7)
    W[0, 4] = np.float16(65504.0)
    W[1, 4] = np.float16(-65504.0)
    W[:, 5] = np.float16(6.1e-5)                  # smallest normal
    # exact ties: with max 7.5 (int4) / 127.5 (int8) the scale is exactly 1
    top = 7.5 if bits == 4 else 127.5
    W[:64, 6] = np.float16(0.5)
    W[0, 6] = np.float16(top)
    W[1, 6] = np.float16(1.5)
    W[2, 6] = np.float16(2.5)
    W[3, 6] = np.float16(-3.5)
    W[4, 6] = np.float16(-top)
    _, _, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
    assert s_ref[0, 6] == np.float16(1.0) and q_ref[1, 6] == 2 and q_ref[2, 6] == 2 and q_ref[3, 6] == -4


def test_quantize_exhaustive_quotient_window():
    """Every (numerator, scale) pair of a dense window goes through the GPU divide/round path."""
    _say("quantize exhaustive window")
    s_vals = np.arange(0x2C00, 0x3000, 8, dtype=np.uint16).view(np.float16)      # 128 scales in [2^-4, 2^-3)
    K = 2048
    N = len(s_vals)
    all16 = np.arange(0x1000, 0x3C00, dtype=np.uint16).view(np.float16)          # positive halves up to 1.0
    W = np.empty((K, N), dtype=np.float16)
    rng = np.random.default_rng(5)
    for j, sj in enumerate(s_vals):
        top = np.float16(float(sj) * 15 / 2.0)
        cand = all16[all16 <= top]
        col = rng.choice(cand, size=K, replace=True)
        col[0] = top
        sign = rng.integers(0, 2, size=K) * 2 - 1
        W[:, j] = (col.astype(np.float32) * sign).astype(np.float16)
    assert_quantizer_parity(W, 4, 0)


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_quantize_quotients_next_to_ties(bits):
    """Numerators chosen next to (k + 1/2) * s for every code k and 256 scales of every mantissa pattern:
    the binary16 values just below and above each tie (two on each side), both signs.  Hundreds of the
    quotients are exact ties (counted below; with binary16 numerators nothing else comes within 2^-13 of
    one), the rest are the closest misses there are: where a product with the reciprocal and the IEEE
    quotient could round differently."""
    _say(f"quantize next to ties int{bits}")
    qmax = (1 << (bits - 1)) - 1
    L = float((1 << bits) - 1)
    tops = np.arange(0x3000, 0x3400, 4, dtype=np.uint16).view(np.float16)         # 256 column maxima in [1/8, 1/4)
    N = len(tops)
    s_col = oracle.scale_from_absmax(tops, bits).astype(np.float64)
    all16 = np.arange(0x0001, 0x3400, dtype=np.uint16).view(np.float16).astype(np.float64)   # ascending
    per_col = 4 * qmax
    K = 128 * (-(-(2 * per_col + 1) // 128))
    W = np.zeros((K, N), dtype=np.float16)
    near = 0
    for n in range(N):
        ties = (np.arange(qmax) + 0.5) * s_col[n]
        at = np.searchsorted(all16, ties)                     # first value >= tie
        idx = np.concatenate([at - 2, at - 1, at, at + 1])
        vals = all16[np.clip(idx, 0, len(all16) - 1)]
        vals = vals[vals <= float(tops[n])]
        quo = (vals.astype(np.float32) / np.float32(s_col[n])).astype(np.float64)
        near += int(np.sum(np.abs(np.abs(quo - np.rint(quo)) - 0.5) < 2.0 ** -13))
        col = np.concatenate([[float(tops[n])], vals, -vals])
        W[: len(col), n] = col.astype(np.float16)
    _say(f"  {near} quotients within 2^-13 of a tie")
    assert near >= 400
    _, _, _, s_ref = assert_quantizer_parity(W, bits, 0)
    assert np.array_equal(s_ref[0].astype(np.float64), s_col)


# ------------------------------------------------------------------ product, oracle-sized cases
def _gemm_case(M, K, N, dtype, bits, g, seed, heavy=False):
    fq = _fq()
    A = workloads.activations(M, K, dtype, seed)
    if heavy:
        W = workloads.weights_heavy_tail(K, N, seed + 1, col_prob=0.02)
    else:
        W = workloads.weights_gaussian(K, N, seed + 1, outlier_prob=1e-3)
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
    C_ref = oracle.gemm_ref(A, q_ref, s_ref)
    Ad = to_dev_act(A, dtype)
    C = from_dev_act(fq.gemm(Ad, codes, scales, bits, g), dtype)
    rel = assert_gemm_close(C, C_ref, dtype, f"M={M} K={K} N={N} {dtype} int{bits} g={g}")
    # determinism: a second call returns the same bits
    C2 = from_dev_act(fq.gemm(Ad, codes, scales, bits, g), dtype)
    assert np.array_equal(C, C2)
    return rel


def test_gemm_config1():
    for bits, g in ((8, 0), (4, 128)):
        _say(f"gemm config1 int{bits} g={g}")
        fq = _fq()
        A, W = workloads.config1(0)
        codes, scales, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
        C = from_dev_act(fq.gemm(to_dev_act(A, "f16"), codes, scales, bits, g), "f16")
        assert_gemm_close(C, oracle.gemm_ref(A, q_ref, s_ref), "f16", "config1")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits,g", [(4, 32), (4, 64), (4, 128), (4, 256), (4, 0), (8, 32), (8, 64), (8, 128), (8, 0)])
@pytest.mark.parametrize("M", [1, 5, 16])
def test_gemm_small_m(dtype, bits, g, M):
    _say(f"gemm small-M {dtype} int{bits} g={g} M={M}")
    # 9 column tiles (ragged against the 4-tile wave groups), 6 k-blocks of 128
    _gemm_case(M, 768, 144, dtype, bits, g, seed=1000 + M + bits + g)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits,g", [(4, 32), (4, 64), (4, 128), (4, 0), (8, 64), (8, 0)])
@pytest.mark.parametrize("M", [17, 40, 130])
def test_gemm_tiled(dtype, bits, g, M):
    _say(f"gemm tiled {dtype} int{bits} g={g} M={M}")
    _gemm_case(M, 768, 304, dtype, bits, g, seed=2000 + M + bits + g)


def _sweep_cases():
    """Seeded draw of (M, K, N, dtype, bits, g): M on both sides of every plan boundary, K from one to a
    few k-blocks (so that the pipelined loops run their prologue, their unrolled body and their tail with
    clamped prefetches), N from one column tile to several ragged column blocks."""
    rng = np.random.default_rng(20240611)
    Ms = [1, 2, 7, 15, 16, 17, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 200, 257, 300]
    cases = []
    for i in range(48):
        bits = int(rng.choice([4, 8]))
        kblk = 128 if bits == 4 else 64
        K = kblk * int(rng.choice([1, 2, 3, 4, 5, 7, 12]))
        N = 16 * int(rng.choice([1, 2, 3, 5, 12, 13, 24, 25, 31, 49]))
        gs = [g for g in (32, 64, 96, 128, 256, 0) if g == 0 or (g <= K and K % g == 0)]
        g = int(rng.choice(gs))
        M = int(Ms[i % len(Ms)])
        dtype = "f16" if rng.integers(2) else "bf16"
        cases.append((M, K, N, dtype, bits, g))
    return cases


@pytest.mark.parametrize("M,K,N,dtype,bits,g", _sweep_cases())
def test_gemm_shape_sweep(M, K, N, dtype, bits, g):
    _say(f"gemm sweep M={M} K={K} N={N} {dtype} int{bits} g={g}")
    _gemm_case(M, K, N, dtype, bits, g, seed=7000 + M + K + N + bits + g)


@pytest.mark.parametrize("dtype,bits,g,M", [("f16", 4, 96, 8), ("bf16", 4, 192, 33), ("f16", 8, 96, 3), ("bf16", 8, 160, 70)])
def test_gemm_group_sizes_that_are_not_powers_of_two(dtype, bits, g, M):
    _say(f"gemm odd group {dtype} int{bits} g={g} M={M}")
    K = 960 * 2 if g in (96, 160, 192) else 768           # 1920 = lcm-friendly: divisible by 96, 160, 192 and 128
    _gemm_case(M, K, 64, dtype, bits, g, seed=3000 + g)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [4, 8])
def test_gemm_heavy_tailed_weights(dtype, bits):
    _say(f"gemm heavy tail {dtype} int{bits}")
    for g in (32, 128, 0):
        for M in (1, 16, 48):
            _gemm_case(M, 1024, 224, dtype, bits, g, seed=4000 + M + g, heavy=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits,g", [(4, 32), (4, 128), (8, 0), (8, 32)])
def test_gemm_one_hot_rows_return_the_dequantised_weights_exactly(dtype, bits, g):
    """A = e_k: no accumulation error, so C must equal q*s rounded once to the output type.

    Every k of two k-blocks is visited, which checks the packed layout element by element."""
    _say(f"gemm one-hot {dtype} int{bits} g={g}")
    fq = _fq()
    K, N = 256, 48
    W = workloads.weights_gaussian(K, N, seed=77 + bits, outlier_prob=0.01)
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
    gg = g or K
    for k0 in range(0, K, 16):
        A = np.zeros((16, K), dtype=np.float32)
        for r in range(16):
            A[r, k0 + r] = 1.0
        A_in = A.astype(np.float16) if dtype == "f16" else A
        C = from_dev_act(fq.gemm(to_dev_act(A_in, dtype), codes, scales, bits, g), dtype)
        for r in range(16):
            k = k0 + r
            expect = round_to_act(q_ref[k].astype(np.float64) * s_ref[k // gg].astype(np.float64), dtype)
            assert np.array_equal(C[r], expect), (k, dtype, bits, g)


def test_gemm_rows_beyond_m_are_not_written():
    _say("gemm guard rows")
    fq = _fq()
    torch = torch_mod()
    K, N, M = 512, 128, 5
    A = workloads.activations(M, K, "f16", 1)
    W = workloads.weights_gaussian(K, N, 2)
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, 4, 128)
    for Mcase in (5, 21):
        A = workloads.activations(Mcase, K, "f16", 1)
        out = torch.full((Mcase + 3, N), 7.0, dtype=torch.float16, device="cuda")
        fq.gemm(to_dev_act(A, "f16"), codes, scales, 4, 128, out=out[:Mcase])
        host = out.cpu().numpy()
        assert np.all(host[Mcase:] == 7.0)
        assert_gemm_close(host[:Mcase].astype(np.float64), oracle.gemm_ref(A, q_ref, s_ref), "f16", "guard")


# ------------------------------------------------------------------ heuristic
def test_choose_group_matches_oracle():
    fq = _fq()
    torch = torch_mod()
    cases = []
    W = workloads.weights_gaussian(1024, 256, 11, outlier_prob=1e-3)
    for alpha in (0.0, 0.3, 0.6, 0.75, 0.9, 0.97, 0.995, 1.0):
        cases.append((W, 256, 64, alpha))
        cases.append((W, 0, 32, alpha))
    Wp = np.full((512, 64), 1.0, dtype=np.float16)
    Wp[:64, 3] = 8.0
    cases += [(Wp, 0, 16, 0.5), (Wp, 0, 16, 0.9), (Wp, 64, 16, 0.5)]
    Wq = np.full((64, 32), 1.0, dtype=np.float16)
    Wq[:32, 1] = 4.0
    cases += [(Wq, 0, 32, 0.5), (Wq, 0, 32, 0.75), (Wq, 0, 32, 0.8)]
    Wo = workloads.weights_gaussian(96 * 4, 32, 5)
    cases += [(Wo, 96, 1, 0.0), (Wo, 0, 32, 0.0), (Wo, 0, 32, 0.4)]
    for W_, gs, gm, alpha in cases:
        _say(f"choose_group K={W_.shape[0]} N={W_.shape[1]} g_start={gs} g_min={gm} alpha={alpha}")
        want = oracle.choose_group(W_, gs, gm, alpha)
        got = fq.choose_group(torch.from_numpy(W_).cuda(), gs, gm, alpha)
        assert got == want, (gs, gm, alpha, got, want)


# ------------------------------------------------------------------ round-trip error (section 3.2)
@pytest.mark.parametrize("K,N", [(32 * 512, 80), (32 * 1024, 48), (32 * 2048, 32), (48 * 256, 272)])
def test_choose_group_deep_halving_trees(K, N):
    """Per-column start with 9, 10, 11 and 8 halving levels (the fold over the levels runs in LDS with 32, 16
    or 64 columns per block, or per column in registers beyond 1024 fine blocks).  One column carries 8.0 in
    its first K / 2^(d+1) rows and 1.0 elsewhere: the halving test then fires at levels 0 .. d and nowhere
    else, so the answer is K / 2^(d+1); plus Gaussian weights at several thresholds."""
    fq = _fq()
    torch = torch_mod()
    f = 48 if K % 48 == 0 and (K // 48) & (K // 48 - 1) == 0 else 32
    levels = (K // f).bit_length() - 1
    assert f << levels == K
    for d in sorted({0, 1, levels // 2, levels - 2, levels - 1}):
        W = np.full((K, N), 1.0, dtype=np.float16)
        W[: K >> (d + 1), N - 3] = 8.0
        want = oracle.choose_group(W, 0, f, 0.5)
        assert want == K >> (d + 1)
        _say(f"choose_group deep K={K} N={N} levels={levels} d={d} -> {want}")
        assert fq.choose_group(torch.from_numpy(W).cuda(), 0, f, 0.5) == want
        assert fq.choose_group(torch.from_numpy(W).cuda(), 0, f, 0.8) == want     # 1 < 0.2 * 8 still holds
        assert fq.choose_group(torch.from_numpy(W).cuda(), 0, f, 0.9) == K        # 1 < 0.1 * 8 does not
        assert oracle.choose_group(W, 0, f, 0.8) == want and oracle.choose_group(W, 0, f, 0.9) == K
    Wg = workloads.weights_gaussian(K, N, 77, outlier_prob=1e-4)
    Wd = torch.from_numpy(Wg).cuda()
    for alpha in (0.2, 0.6, 0.9, 0.99):
        want = oracle.choose_group(Wg, 0, f, alpha)
        _say(f"choose_group deep gaussian K={K} alpha={alpha} -> {want}")
        assert fq.choose_group(Wd, 0, f, alpha) == want


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("K,N,g", [(384, 80, 32), (512, 272, 64), (1024, 16, 0), (256, 1040, 256), (768, 304, 128)])
def test_quant_error_matches_oracle(bits, K, N, g):
    _say(f"quant error int{bits} K={K} N={N} g={g}")
    fq = _fq()
    torch = torch_mod()
    W = workloads.weights_gaussian(K, N, 90 + K + N, outlier_prob=2e-3)
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
    sse, mx = fq.quant_error(torch.from_numpy(W).cuda(), codes, scales, bits, g)
    sse_ref, mx_ref = oracle.quant_error(W, q_ref, s_ref)
    assert mx == mx_ref                                   # one exact difference: bit-exact
    # both sides add the same exactly rounded squares, in different orders: K * N <= 3e5 terms of
    # relative rounding 2^-53 each
    assert abs(sse - sse_ref) <= 1e-11 * sse_ref, (sse, sse_ref)
    sse2, mx2 = fq.quant_error(torch.from_numpy(W).cuda(), codes, scales, bits, g)
    assert (sse2, mx2) == (sse, mx)                       # deterministic


def test_quant_error_heavy_tail_and_zero_matrix():
    fq = _fq()
    torch = torch_mod()
    W = workloads.weights_heavy_tail(512, 96, seed=17)
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, 4, 64)
    sse, mx = fq.quant_error(torch.from_numpy(W).cuda(), codes, scales, 4, 64)
    sse_ref, mx_ref = oracle.quant_error(W, q_ref, s_ref)
    assert mx == mx_ref and abs(sse - sse_ref) <= 1e-11 * sse_ref
    Z = np.zeros((256, 32), dtype=np.float16)
    codes, scales, _, _ = assert_quantizer_parity(Z, 8, 128)
    assert fq.quant_error(torch.from_numpy(Z).cuda(), codes, scales, 8, 128) == (0.0, 0.0)


# ------------------------------------------------------------------ grouped (mixture of experts)
@pytest.mark.parametrize("dtype,bits,g", [("f16", 4, 64), ("bf16", 4, 64), ("f16", 8, 0)])
def test_grouped_gemm_small(dtype, bits, g):
    _say(f"grouped small {dtype} int{bits} g={g}")
    fq = _fq()
    torch = torch_mod()
    E, K, N = 6, 256, 96
    rows = [70, 0, 1, 16, 130, 0]
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    A = workloads.activations(int(offsets[-1]), K, dtype, 8)
    qs, ss, codes_l, scales_l = [], [], [], []
    for e in range(E):
        W = workloads.weights_gaussian(K, N, 50 + e, outlier_prob=1e-3)
        c, s, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
        codes_l.append(c)
        scales_l.append(s.reshape(-1))
        qs.append(q_ref)
        ss.append(s_ref)
    codes = torch.cat(codes_l)
    scales = torch.cat(scales_l)
    out = torch.full((int(offsets[-1]), N), 3.0, dtype=torch.float16 if dtype == "f16" else torch.bfloat16, device="cuda")
    fq.gemm_grouped(to_dev_act(A, dtype), offsets.tolist(), codes, scales, bits, g, N, out=out)
    C = from_dev_act(out, dtype)
    C_ref = oracle.gemm_ref_grouped(A, offsets, qs, ss)
    assert_gemm_close(C, C_ref, dtype, "grouped")
    for e in range(E):
        if rows[e]:
            sl = slice(offsets[e], offsets[e + 1])
            assert_gemm_close(C[sl], C_ref[sl], dtype, f"expert {e}")


def _grouped_case(dtype, bits, g, K, N, rows, seed, shared_weights=False):
    """Experts with the given row counts; returns nothing, asserts parity per expert."""
    fq = _fq()
    torch = torch_mod()
    E = len(rows)
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    A = workloads.activations(int(offsets[-1]), K, dtype, seed)
    qs, ss, codes_l, scales_l = [], [], [], []
    for e in range(E):
        if e == 0 or not shared_weights:
            W = workloads.weights_gaussian(K, N, seed + 50 + e, outlier_prob=1e-3)
            c, s, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
        codes_l.append(c)
        scales_l.append(s.reshape(-1))
        qs.append(q_ref)
        ss.append(s_ref)
    codes = torch.cat(codes_l)
    scales = torch.cat(scales_l)
    out = torch.full((int(offsets[-1]), N), 3.0, dtype=torch.float16 if dtype == "f16" else torch.bfloat16, device="cuda")
    fq.gemm_grouped(to_dev_act(A, dtype), offsets.tolist(), codes, scales, bits, g, N, out=out)
    C = from_dev_act(out, dtype)
    C_ref = oracle.gemm_ref_grouped(A, offsets, qs, ss)
    for e in range(E):
        if rows[e]:
            sl = slice(offsets[e], offsets[e + 1])
            assert_gemm_close(C[sl], C_ref[sl], dtype, f"expert {e} ({rows[e]} rows)")


@pytest.mark.parametrize("dtype,bits,g", [("f16", 4, 64), ("bf16", 4, 128), ("bf16", 8, 32), ("f16", 8, 0),
                                          ("f16", 4, 128), ("bf16", 4, 64), ("f16", 4, 0)])
def test_grouped_gemm_tile_boundaries(dtype, bits, g):
    """Row counts on both sides of every row-tile size (32 / 64 / 128) and several column blocks with a
    ragged last one for both the 4-wave (192 columns) and the 8-wave (384 columns) block shapes."""
    _say(f"grouped tile boundaries {dtype} int{bits} g={g}")
    _grouped_case(dtype, bits, g, 256, 400, [32, 33, 64, 65, 128, 129, 0, 193, 40, 161, 1], seed=31)


@pytest.mark.parametrize("dtype,bits,g", [("f16", 4, 64), ("bf16", 4, 128), ("f16", 8, 0), ("bf16", 3, 64)])
def test_grouped_gemm_wide_matrix_uses_eight_wave_blocks_for_every_tile_size(dtype, bits, g):
    """49 column tiles: two full 8-wave column blocks and one with a single tile, for the 32-, 64- and
    128-row tiles alike."""
    _say(f"grouped wide {dtype} int{bits} g={g}")
    _grouped_case(dtype, bits, g, 256, 784, [31, 33, 64, 0, 130, 1, 97], seed=33)


def test_grouped_gemm_more_tiles_than_one_launch_holds():
    """260 row tiles of 128 rows: the by-value tile list holds 256, so a second launch takes the rest."""
    _say("grouped 130 experts x 256 rows")
    _grouped_case("f16", 4, 128, 128, 48, [256] * 130, seed=32, shared_weights=True)


# ------------------------------------------------------------------ bf16 activations on the fp16 matrix path
def _rows_case(M, K, N, bits, g, seed, row_scales):
    """bf16 activations whose rows are scaled by `row_scales` (wide matrix, 128-row blocks: the rows are
    rewritten as binary16 over a power of two per row); parity per row, relative to that row's largest output."""
    fq = _fq()
    W = workloads.weights_gaussian(K, N, seed, outlier_prob=1e-3)
    A = workloads.activations(M, K, "bf16", seed + 1).astype(np.float64)
    A *= np.asarray(row_scales, dtype=np.float64)[:, None]
    A = workloads.round_to_bf16(A.astype(np.float32))
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, bits, g)
    assert fq.gemm_workspace_bytes_for(M, N, K, bits, g, fq.FQ_BF16) > fq.gemm_workspace_bytes_for(M, N, K, bits, g, fq.FQ_F16)
    C = from_dev_act(fq.gemm(to_dev_act(A, "bf16"), codes, scales, bits, g), "bf16")
    C_ref = oracle.gemm_ref(A, q_ref, s_ref)
    assert np.all(np.isfinite(C))
    for r in range(M):
        top = np.max(np.abs(C_ref[r]))
        err = np.max(np.abs(C[r] - C_ref[r]))
        assert err <= TOL["bf16"] * top, f"row {r} (scale {row_scales[r]:.3g}): {err} > {TOL['bf16']} * {top}"


@pytest.mark.parametrize("bits,g", [(4, 128), (4, 64), (8, 0), (3, 32)])
def test_gemm_bf16_rows_rewritten_as_binary16(bits, g):
    _say(f"bf16 via fp16 path int{bits} g={g}")
    M, K, N = 270, 256, 8192            # more than 256 rows: 128-row blocks
    rng = np.random.default_rng(77)
    row_scales = 2.0 ** rng.integers(-60, 60, size=M).astype(np.float64)
    row_scales[0] = 0.0                 # an all-zero row
    row_scales[1] = 2.0 ** -120         # far below the binary16 range
    row_scales[2] = 2.0 ** 110          # far above it
    row_scales[3] = 1.0
    _rows_case(M, K, N, bits, g, 9100 + bits + g, row_scales)


def test_gemm_bf16_rows_with_outliers_inside_a_row():
    """One element 2^20 times larger than the rest of its row: the small elements keep their relative
    precision (they are still normal binary16 numbers after the row's division)."""
    _say("bf16 via fp16 path, outlier inside rows")
    fq = _fq()
    M, K, N = 260, 384, 8192
    W = workloads.weights_gaussian(K, N, 9200, outlier_prob=1e-3)
    A = workloads.activations(M, K, "bf16", 9201).astype(np.float32)
    A[:, 5] *= np.float32(2.0 ** 20)
    A = workloads.round_to_bf16(A)
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, 4, 128)
    assert fq.gemm_workspace_bytes_for(M, N, K, 4, 128, fq.FQ_BF16) > fq.gemm_workspace_bytes_for(M, N, K, 4, 128, fq.FQ_F16)
    C = from_dev_act(fq.gemm(to_dev_act(A, "bf16"), codes, scales, 4, 128), "bf16")
    assert_gemm_close(C, oracle.gemm_ref(A, q_ref, s_ref), "bf16", "outlier column")
    # without the outlier column the same rows: the small elements alone must still be accurate
    A2 = A.copy()
    A2[:, 5] = 0
    C2 = from_dev_act(fq.gemm(to_dev_act(A2, "bf16"), codes, scales, 4, 128), "bf16")
    assert_gemm_close(C2, oracle.gemm_ref(A2, q_ref, s_ref), "bf16", "rows without the outlier")


def test_gemm_bf16_wide_matrix_split_k_and_tail():
    """Wide matrices whose plans split K (uniformly, or for the tail round only) on the fp16 path."""
    _say("bf16 via fp16 path with split K")
    fq = _fq()
    for M, K, N in ((384, 2048, 8192), (300, 1024, 12288)):
        assert fq.gemm_workspace_bytes_for(M, N, K, 4, 128, fq.FQ_BF16) > fq.gemm_workspace_bytes_for(M, N, K, 4, 128, fq.FQ_F16)
        _say("  " + fq.gemm_describe(M, N, K, 4, 128))
        _gemm_case(M, K, N, "bf16", 4, 128, seed=9300 + M)


@pytest.mark.parametrize("M,K,N,dtype,g", [(300, 4224, 6160, "f16", 128), (260, 4224, 6160, "bf16", 0),
                                           (1100, 1152, 6160, "f16", 0), (900, 1152, 12288, "bf16", 128),
                                           (1030, 1280, 9232, "f16", 256), (300, 4224, 6160, "f16", 64),
                                           (600, 128, 12288, "f16", 128)])
def test_gemm_int8_two_layout_blocks_per_k_block(M, K, N, dtype, g):
    """8-bit codes in the 128-row, 8-wave shape: the kernel takes two 64-row k-blocks of the packed layout
    per k-block when K is a multiple of 128 and the group size too (checked through the plan's k-block
    count: K / 128 instead of K / 64 blocks in all); an odd number of them, a ragged split of K, ragged
    last row blocks, the fp16 path for bf16 rows (N >= 8192), a single k-block, and g = 64, which keeps
    the 64-row blocks."""
    import re
    fq = _fq()
    desc = fq.gemm_describe(M, N, K, 8, g)
    _say(f"int8 wide M={M} K={K} N={N} {dtype} g={g}: {desc}")
    m = re.match(r"tiled mt=8 waves=8 splits=(\d+) kb_per_split=(\d+)", desc)
    assert m, desc
    splits, kbs = int(m.group(1)), int(m.group(2))
    unit = 128 if (g or K) % 128 == 0 else 64
    assert kbs * splits >= K // unit > kbs * (splits - 1)
    _gemm_case(M, K, N, dtype, 8, g, seed=9500 + M + g)


@pytest.mark.parametrize("dtype,g,K", [("bf16", 128, 384), ("f16", 0, 640), ("f16", 64, 384)])
def test_grouped_gemm_int8_two_layout_blocks_per_k_block(dtype, g, K):
    """8-bit experts: the 128-row tiles take two 64-row layout k-blocks per k-block when K and the group size
    are multiples of 128 (an odd number of them here), the smaller tiles and g = 64 keep the 64-row blocks."""
    _say(f"grouped int8 wide {dtype} g={g} K={K}")
    _grouped_case(dtype, 8, g, K, 784, [130, 31, 64, 0, 257, 1, 97], seed=35)
