"""Seeded random shapes through every product entry point against the oracle.

The other GPU tests pick their shapes by hand (plan boundaries, ragged tiles, full sizes); this one draws
M, N, K, the group size, the code width, the activation type, the weight spread and the entry point at random
(fixed seed), so that combinations nobody thought of are compared as well.  Codes are compared bit by bit, the
products within the tolerance of the activation type.
"""
import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads

from gpu_util import TOL, from_dev_act, to_dev_act, torch_mod

pytestmark = pytest.mark.gpu

CASES = 96


def _draw(rng):
    kind = str(rng.choice(["gemm", "gemm", "gemm", "grouped", "w4a8", "bf16_scales"]))
    bits = 4 if kind == "w4a8" else int(rng.choice([3, 4, 4, 8]))
    kblk = 64 if bits == 8 else 128
    K = kblk * int(rng.integers(1, 2048 // kblk + 1))
    N = 16 * int(rng.integers(1, 160))
    M = int(rng.integers(1, int(rng.choice([16, 40, 140, 300, 700])) + 1))
    gs = [g for g in range(32, K + 1, 32) if K % g == 0]
    g = int(rng.choice(gs + [0, 128 if K % 128 == 0 else gs[0]]))
    dtype = "bf16" if kind == "bf16_scales" else str(rng.choice(["f16", "bf16"]))
    sigma = float(rng.choice([0.02, 1.0, 1e-3]))
    outliers = float(rng.choice([0.0, 1e-3, 1e-2]))
    seeds = [int(x) for x in rng.integers(1 << 30, size=8)]
    return kind, bits, M, N, K, g, dtype, sigma, outliers, seeds


@pytest.mark.parametrize("chunk", range(4))
def test_random_shapes_match_oracle(chunk):
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    rng = np.random.default_rng(20230817 + chunk)
    for case in range(CASES // 4):
        kind, bits, M, N, K, g, dtype, sigma, outliers, seeds = _draw(rng)
        what = f"chunk {chunk} case {case}: {kind} bits={bits} M={M} N={N} K={K} g={g} {dtype} sigma={sigma}"
        print("  " + what, flush=True)
        W = workloads.weights_gaussian(K, N, seed=seeds[0], sigma=sigma, outlier_prob=outliers)
        A = workloads.activations(M, K, dtype, seeds[1])
        Ad = to_dev_act(A, dtype)
        if kind in ("gemm", "bf16_scales"):
            sf = "bf16" if kind == "bf16_scales" else "f16"
            q_ref, s_ref = oracle.quantize(W, bits, g, sf)
            codes, scales = fq.quantize(torch.from_numpy(W).cuda(), bits, g,
                                        fq.FQ_SCALE_BF16 if sf == "bf16" else fq.FQ_SCALE_F16)
            assert np.array_equal(fq.unpack(codes, K, N, bits).cpu().numpy(), q_ref), what + ": codes differ"
            C = from_dev_act(fq.gemm(Ad, codes, scales, bits, g), dtype)
            C_ref = oracle.gemm_ref(A, q_ref, s_ref)
        elif kind == "grouped":
            E = 1 + seeds[2] % 5
            cuts = np.sort(np.random.default_rng(seeds[3]).integers(0, M + 1, E - 1))
            offsets = np.concatenate([[0], cuts, [M]]).astype(np.int32)
            qs, ss, cl, sl = [], [], [], []
            for e in range(E):
                We = workloads.weights_gaussian(K, N, seed=seeds[4] + e, sigma=sigma)
                q_ref, s_ref = oracle.quantize(We, bits, g)
                c, s = fq.quantize(torch.from_numpy(We).cuda(), bits, g)
                qs.append(q_ref); ss.append(s_ref); cl.append(c); sl.append(s)
            C = from_dev_act(fq.gemm_grouped(Ad, offsets.tolist(), torch.stack(cl).contiguous(),
                                             torch.stack(sl).contiguous(), bits, g, N), dtype)
            C_ref = oracle.gemm_ref_grouped(A, offsets, qs, ss)
        else:
            q_ref, z_ref, t_ref = oracle.quantize_int_scales(W, g)
            codes, z, t = fq.quantize_w4a8(torch.from_numpy(W).cuda(), g)
            assert np.array_equal(fq.unpack_w4a8(codes, K, N).cpu().numpy(), q_ref), what + ": codes differ"
            assert np.array_equal(z.cpu().numpy(), z_ref), what + ": multipliers differ"
            Aq, alpha = fq.quantize_act_i8(Ad)
            a_ref, alpha_ref = oracle.quantize_activations_int8(A)
            assert np.array_equal(Aq.cpu().numpy(), a_ref), what + ": int8 activations differ"
            out_dt = torch.float16 if dtype == "f16" else torch.bfloat16
            C = from_dev_act(fq.gemm_w4a8(Aq, alpha, codes, z, t, g, out_dt), dtype)
            _, C_ref = oracle.gemm_ref_int(a_ref, alpha_ref, q_ref, z_ref, t_ref)
        scale = np.max(np.abs(C_ref))
        err = np.max(np.abs(C - C_ref))
        assert np.isfinite(C).all(), what + ": non-finite output"
        assert err <= TOL[dtype] * scale, f"{what}: max err {err:.4g} > {TOL[dtype]} * {scale:.4g}"
