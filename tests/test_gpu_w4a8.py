"""GPU parity of the integer path (int8 activations x int4 weights with integer group scales) with its oracle.

Bit-exact: the weight codes, the multipliers z, the column steps t, the int8 activations and their scales.
The product's integer sums are exact on both sides, so the output may differ from the oracle's
alpha * t * S only by the binary32 evaluation of that scaling and the rounding to the output type: checked
element by element against the correctly rounded oracle value with one unit of slack, and against the
tolerance of the floating-point path.
"""
import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads

from gpu_util import TOL, from_dev_act, round_to_act, to_dev_act, torch_mod

pytestmark = pytest.mark.gpu


def _quantize_weights(W, g):
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N = W.shape
    codes, z, t = fq.quantize_w4a8(torch.from_numpy(W).cuda(), g)
    q_ref, z_ref, t_ref = oracle.quantize_int_scales(W, g)
    assert np.array_equal(t.view(torch.int16).cpu().numpy().view(np.uint16), t_ref.view(np.uint16)), "column steps differ"
    assert np.array_equal(z.cpu().numpy(), z_ref), "multipliers differ"
    assert np.array_equal(fq.unpack_w4a8(codes, K, N).cpu().numpy(), q_ref), "codes differ"
    return codes, z, t, q_ref, z_ref, t_ref


def _quantize_acts(A, dtype):
    from paper_2308_09723_amd import fq
    Aq, alpha = fq.quantize_act_i8(to_dev_act(A, dtype))
    a_ref, alpha_ref = oracle.quantize_activations_int8(A)
    assert np.array_equal(alpha.cpu().numpy().view(np.uint32), alpha_ref.view(np.uint32)), "activation scales differ"
    assert np.array_equal(Aq.cpu().numpy(), a_ref), "int8 activations differ"
    return Aq, alpha, a_ref, alpha_ref


def _check_product(C, C_ref, dtype, what):
    """C: float64 view of the GPU result; C_ref: the oracle's exact alpha * t * S in float64."""
    scale = np.max(np.abs(C_ref))
    err = np.max(np.abs(C - C_ref))
    assert err <= TOL[dtype] * scale, f"{what}: {err} > {TOL[dtype]} * {scale}"
    # element by element: the correctly rounded value, or its neighbour (the scaling runs in binary32)
    want = round_to_act(C_ref, dtype)
    ulp = np.maximum(np.abs(want), np.float64(2.0 ** -14 if dtype == "f16" else 2.0 ** -120)) * (2.0 ** -10 if dtype == "f16" else 2.0 ** -7)
    bad = np.abs(C - want) > ulp
    assert not bad.any(), f"{what}: {int(bad.sum())} elements further than one unit from the rounded oracle value"
    return err / scale if scale > 0 else 0.0


def test_weight_quantiser_special_values():
    """Zero groups and columns, subnormals, +-65504, exact ties, groups of very different widths."""
    rng = np.random.default_rng(5)
    K, N = 256, 64
    W = (rng.standard_normal((K, N)) * 0.05).astype(np.float16)
    W[:32, 0] = 0
    W[:, 1] = 0
    W[:32, 2] = np.float16(6e-8)
    W[32:, 2] *= np.float16(1e-3)
    W[5, 3] = np.float16(65504.0)
    W[140, 3] = np.float16(-65504.0)
    W[64:96, 4] = (W[64:96, 4].astype(np.float32) * 1e-3).astype(np.float16)
    W[:, 5] = np.float16(0.75)
    W[:, 6] = 0
    W[0, 6] = np.float16(3.75)
    W[32, 6] = np.float16(0.46875)
    W[33, 6] = np.float16(1.5 * 2 ** -4)
    W[34, 6] = np.float16(2.5 * 2 ** -4)
    W[35, 6] = np.float16(-0.5 * 2 ** -4)
    W[:, 7] = np.float16(6e-8)                        # a column of the smallest subnormal
    for g in (32, 64, 128, 0):
        _quantize_weights(W, g)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_activation_quantiser(dtype):
    rng = np.random.default_rng(8)
    M, K = 37, 1024
    A = workloads.activations(M, K, dtype, 61).astype(np.float32)
    A[1] = 0
    A[2, 7] = -65504.0 if dtype == "f16" else -3.0e38
    A[3] *= 2.0 ** -10
    A[4, :] = 0.5
    A[4, 3] = 63.75                                   # alpha = 0.5 exactly: quotients 1.0 and 127.5
    A[5, rng.integers(0, K, 50)] *= 40.0
    A = A.astype(np.float16) if dtype == "f16" else workloads.round_to_bf16(A)
    _quantize_acts(A, dtype)


@pytest.mark.parametrize("K", [8, 1000, 1003, 12288 + 40, 7])
def test_activation_quantiser_row_lengths(K):
    """Rows of whole 16-byte units (eight values per lane), rows that are not (one value per lane), rows shorter
    than a block."""
    for dtype in ("f16", "bf16"):
        _quantize_acts(workloads.activations(9, K, dtype, 700 + K), dtype)


@pytest.mark.parametrize("g", [32, 64, 96, 128, 0])
@pytest.mark.parametrize("M,dtype", [(1, "f16"), (5, "bf16"), (16, "f16"), (24, "bf16"), (50, "f16"), (130, "bf16"),
                                     (300, "f16")])
def test_product_matches_oracle(M, dtype, g):
    """Every block height (16 / 32 / 64 / 128 rows), ragged row and column blocks, K split over the grid or not,
    every multiplier-row pattern (g = 32, 64, 96 = does not divide a k-block, 128, K)."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N = 768, 1200 - 1200 % 16                      # 75 column tiles: ragged against 24-tile blocks
    W = workloads.weights_gaussian(K, N, seed=70 + (g or 1), outlier_prob=2e-3)
    codes, z, t, q_ref, z_ref, t_ref = _quantize_weights(W, g)
    A = workloads.activations(M, K, dtype, 80 + M)
    Aq, alpha, a_ref, alpha_ref = _quantize_acts(A, dtype)
    out_dt = torch.float16 if dtype == "f16" else torch.bfloat16
    C = from_dev_act(fq.gemm_w4a8(Aq, alpha, codes, z, t, g, out_dt), dtype)
    S_ref, C_ref = oracle.gemm_ref_int(a_ref, alpha_ref, q_ref, z_ref, t_ref)
    rel = _check_product(C, C_ref, dtype, f"M={M} g={g}")
    print(f"  w4a8 M={M} {dtype} g={g or K}: rel err {rel:.2e}", flush=True)


@pytest.mark.parametrize("M,K,N,g", [(7, 4096, 192, 64), (16, 8192, 48, 128), (3, 2048, 1040, 0), (1, 128, 16, 128),
                                     (12, 1536, 6000, 96)])
def test_small_m_block_shapes(M, K, N, g):
    """The small-M kernel of the integer path on shapes that drive its plan to its corners: few column tiles
    (K split over the grid, int32 slabs summed by the second kernel), a single tile and a single k-block, one group
    per column, many column groups per block, two activation units per lane (M = 16 with one column group)."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    N -= N % 16
    W = workloads.weights_gaussian(K, N, seed=300 + M, outlier_prob=2e-3)
    codes, z, t, q_ref, z_ref, t_ref = _quantize_weights(W, g)
    for dtype in ("f16", "bf16"):
        A = workloads.activations(M, K, dtype, 310 + M)
        Aq, alpha, a_ref, alpha_ref = _quantize_acts(A, dtype)
        out_dt = torch.float16 if dtype == "f16" else torch.bfloat16
        C = from_dev_act(fq.gemm_w4a8(Aq, alpha, codes, z, t, g, out_dt), dtype)
        _, C_ref = oracle.gemm_ref_int(a_ref, alpha_ref, q_ref, z_ref, t_ref)
        _check_product(C, C_ref, dtype, f"small-M M={M} K={K} N={N} g={g}")


def test_product_extreme_sums_and_one_hot_rows():
    """All activations +-127 against all codes -7 with z = 16 (the largest sums), and one-hot activation rows
    that read back single rows of q * z (every row of two k-blocks)."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N = 4096, 256
    W = np.full((K, N), -0.5, dtype=np.float16)
    W[:, ::2] = np.float16(0.5)
    codes, z, t, q_ref, z_ref, t_ref = _quantize_weights(W, 128)
    assert np.all(z_ref == 16) and np.all(np.abs(q_ref) == 7)
    A = np.full((3, K), 2.0, dtype=np.float16)
    A[1] = np.float16(-2.0)
    A[2, ::3] = np.float16(-2.0)
    Aq, alpha, a_ref, alpha_ref = _quantize_acts(A, "f16")
    assert np.all(np.abs(a_ref) == 127)
    C = from_dev_act(fq.gemm_w4a8(Aq, alpha, codes, z, t, 128, torch.float16), "f16")
    S_ref, C_ref = oracle.gemm_ref_int(a_ref, alpha_ref, q_ref, z_ref, t_ref)
    assert int(np.abs(S_ref).max()) == K * 127 * 112
    _check_product(C, C_ref, "f16", "extreme sums")
    # one-hot rows
    K2, N2 = 256, 64
    W2 = workloads.weights_gaussian(K2, N2, seed=77, outlier_prob=1e-2)
    codes2, z2, t2, q2, zr2, tr2 = _quantize_weights(W2, 32)
    A2 = np.zeros((K2, K2), dtype=np.float16)
    A2[np.arange(K2), np.arange(K2)] = np.float16(1.0)
    Aq2, alpha2, a2, al2 = _quantize_acts(A2, "f16")
    C2 = from_dev_act(fq.gemm_w4a8(Aq2, alpha2, codes2, z2, t2, 32, torch.float16), "f16")
    _, C2_ref = oracle.gemm_ref_int(a2, al2, q2, zr2, tr2)
    _check_product(C2, C2_ref, "f16", "one-hot rows")


@pytest.mark.parametrize("layer", ["out_proj", "qkv"])
def test_full_size_layer_on_sampled_columns(layer):
    """The out-proj- and QKV-shaped layers (the latter is the one bench.py times for this path) at M = 8 and
    M = 2048, on a column sample that covers every 384-column block."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    W = workloads.opt175b_weight(layer, seed=9)
    K, N = W.shape
    cols = np.unique(np.concatenate([np.arange(0, N, 384) + (np.arange(0, N, 384) // 384 * 37) % 384, [0, 15, N - 16, N - 1]]))
    cols = cols[cols < N]
    cols_d = torch.from_numpy(cols).cuda()
    codes, z, t = fq.quantize_w4a8(torch.from_numpy(W).cuda(), 128)
    q_ref, z_ref, t_ref = oracle.quantize_int_scales(np.ascontiguousarray(W[:, cols]), 128)
    assert np.array_equal(fq.unpack_w4a8(codes, K, N).index_select(1, cols_d).cpu().numpy(), q_ref)
    assert np.array_equal(z.index_select(1, cols_d).cpu().numpy(), z_ref)
    assert np.array_equal(t.index_select(0, cols_d).view(torch.int16).cpu().numpy().view(np.uint16), t_ref.view(np.uint16))
    for M, dtype in ((8, "f16"), (2048, "bf16")):
        A = workloads.activations(M, K, dtype, 90 + M)
        Aq, alpha, a_ref, alpha_ref = _quantize_acts(A, dtype)
        out_dt = torch.float16 if dtype == "f16" else torch.bfloat16
        Cd = fq.gemm_w4a8(Aq, alpha, codes, z, t, 128, out_dt)
        assert bool(torch.isfinite(Cd.float()).all())
        C = from_dev_act(Cd.index_select(1, cols_d), dtype)
        _, C_ref = oracle.gemm_ref_int(a_ref, alpha_ref, q_ref, z_ref, t_ref)
        rel = _check_product(C, C_ref, dtype, f"{layer} M={M}")
        print(f"  w4a8 {layer} M={M} {dtype}: rel err {rel:.2e}", flush=True)


def test_rejects_bad_arguments():
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    x = torch.zeros(64, dtype=torch.uint8, device="cuda")
    p = x.data_ptr()
    assert fq.quantize_w4a8_raw(p, 1024, 1000, 128, p, p, p, 0) == fq.FQ_ERR_UNSUPPORTED      # N % 16
    assert fq.quantize_w4a8_raw(p, 1024, 1024, 100, p, p, p, 0) == fq.FQ_ERR_INVALID_ARG      # g does not divide K
    assert fq.quantize_w4a8_raw(p, 262144, 1024, 128, p, p, p, 0) == fq.FQ_ERR_UNSUPPORTED    # K beyond the int32 bound
    assert fq.quantize_w4a8_raw(None, 1024, 1024, 128, p, p, p, 0) == fq.FQ_ERR_INVALID_ARG
    assert fq.quantize_act_i8_raw(p, 7, 4, 1024, p, p, 0) == fq.FQ_ERR_INVALID_ARG
    assert fq.gemm_w4a8_raw(p, p, 4, 1024, 1024, p, p, p, 128, p, 3, p, 64, 0) == fq.FQ_ERR_INVALID_ARG
    assert fq.gemm_w4a8_raw(p, p, 0, 1024, 1024, p, p, p, 128, p, 0, None, 0, 0) == fq.FQ_OK
    need = fq.gemm_w4a8_workspace_bytes(4, 1024, 4096, 128)
    assert need > 0 and need % (4 * 1024 * 4) == 0           # whole slabs of int32 partial sums
    assert fq.gemm_w4a8_raw(p, p, 4, 1024, 4096, p, p, p, 128, p, 0, None, 0, 0) == fq.FQ_ERR_WORKSPACE
