"""Helpers shared by the GPU parity tests: host<->device plumbing and the oracle-side reference."""
import numpy as np

import oracle
from paper_2308_09723_amd import workloads

TOL = {"f16": 4e-3, "bf16": 1.6e-2}   # max|C - C_ref| <= tol * max|C_ref|


def torch_mod():
    import torch
    return torch


def to_dev_act(A, dtype):
    """numpy activations (float16 array, or float32 array of bf16 values) -> cuda tensor."""
    torch = torch_mod()
    if dtype == "f16":
        return torch.from_numpy(np.ascontiguousarray(A)).cuda()
    bits = workloads.bf16_bits(A).view(np.int16)
    return torch.from_numpy(bits).cuda().view(torch.bfloat16)


def from_dev_act(C, dtype):
    """cuda result -> float64 numpy."""
    torch = torch_mod()
    if dtype == "f16":
        return C.cpu().numpy().astype(np.float64)
    bits = C.view(torch.int16).cpu().numpy().view(np.uint16)
    return workloads.bf16_from_bits(bits).astype(np.float64)


def round_to_act(x64, dtype):
    """float64 -> nearest value of the activation type (as float64)."""
    if dtype == "f16":
        return x64.astype(np.float16).astype(np.float64)
    return workloads.round_to_bf16(x64.astype(np.float32)).astype(np.float64)


def gpu_quantize(W, bits, g):
    """Quantise on the GPU; returns (codes, scales) device tensors plus host copies of q and scale bits."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    Wd = torch.from_numpy(W).cuda()
    codes, scales = fq.quantize(Wd, bits, g)
    K, N = W.shape
    q = fq.unpack(codes, K, N, bits).cpu().numpy()
    s_bits = scales.view(torch.int16).cpu().numpy().view(np.uint16)
    return codes, scales, q, s_bits


def assert_quantizer_parity(W, bits, g):
    q_ref, s_ref = oracle.quantize(W, bits, g)
    codes, scales, q, s_bits = gpu_quantize(W, bits, g)
    assert np.array_equal(s_bits, s_ref.view(np.uint16)), "scales differ"
    assert np.array_equal(q, q_ref), "codes differ"
    return codes, scales, q_ref, s_ref


def assert_gemm_close(C, C_ref, dtype, what=""):
    scale = np.max(np.abs(C_ref))
    err = np.max(np.abs(C - C_ref))
    assert err <= TOL[dtype] * scale, f"{what}: max err {err:.4g} > {TOL[dtype]} * {scale:.4g}"
    return err / scale if scale > 0 else 0.0
