"""The product under HIP graph capture: fq_gemm only launches kernels (no memset, no allocation), so a
captured sequence must replay correctly any number of times.  Each replay is compared with the eager
result for the inputs of that replay, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads

from gpu_util import assert_gemm_close, assert_quantizer_parity, from_dev_act, to_dev_act, torch_mod

pytestmark = pytest.mark.gpu


def test_captured_products_replay_correctly():
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N = 768, 304
    W = workloads.weights_gaussian(K, N, 77, outlier_prob=1e-3)
    codes, scales, q_ref, s_ref = assert_quantizer_parity(W, 4, 128)
    shapes = [(1, "f16"), (8, "f16"), (40, "bf16"), (130, "bf16")]     # small-M, small-M, tiled + split-K, tiled
    bufs = []
    for M, dtype in shapes:
        A = to_dev_act(workloads.activations(M, K, dtype, 5 + M), dtype)
        C = torch.zeros((M, N), dtype=A.dtype, device="cuda")
        need = fq.gemm_workspace_bytes(M, N, K, 4, 128)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        bufs.append((M, dtype, A, C, ws))

    def run_all(stream):
        for M, dtype, A, C, ws in bufs:
            st = fq.gemm_raw(A.data_ptr(), fq.FQ_F16 if dtype == "f16" else fq.FQ_BF16, M, N, K, codes.data_ptr(),
                             scales.data_ptr(), 4, 128, C.data_ptr(), ws.data_ptr(), ws.numel(), stream)
            assert st == fq.FQ_OK

    # first calls outside capture (one-time kernel attributes are set on first use)
    run_all(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run_all(torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        new_inputs = []
        for M, dtype, A, C, ws in bufs:
            host = workloads.activations(M, K, dtype, 100 * rep + M)
            A.copy_(to_dev_act(host, dtype))
            C.fill_(7.0)
            new_inputs.append(host)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (M, dtype, A, C, ws), host in zip(bufs, new_inputs):
            got = from_dev_act(C, dtype)
            assert_gemm_close(got, oracle.gemm_ref(host, q_ref, s_ref), dtype, f"replay {rep} M={M}")
            eager = from_dev_act(fq.gemm(A, codes, scales, 4, 128), dtype)      # eager work between replays
            assert np.array_equal(got, eager), f"replay {rep} M={M}: differs from the eager result"
