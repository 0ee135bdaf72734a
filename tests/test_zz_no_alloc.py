"""fq_gemm_noalloc (the entry point for callers that cannot allocate: its scratch is a device array inside
the library) against fq_gemm on the same inputs, through the C ABI.  Both run the same kernels, so the
results must be bit-identical.  Every case makes two calls in a row, the second with a smaller input, on
shapes whose plans use the scratch: split-K partial sums of the small-M kernel and of the tiled kernel, and
bfloat16 rows rewritten as binary16.  (Plans that split a partly filled last round of blocks along K need
more than the static scratch holds at any size: those must be refused.)"""
import numpy as np
import pytest

from paper_2308_09723_amd import workloads

from gpu_util import torch_mod

pytestmark = pytest.mark.gpu


def _pair(fq, torch, W_codes, scales, K, N, bits, g, M, dtype, seed):
    act = fq.FQ_F16 if dtype == "f16" else fq.FQ_BF16
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    A = workloads.activations(M, K, dtype, seed)
    if dtype == "f16":
        Ad = torch.from_numpy(A).cuda()
    else:
        Ad = torch.from_numpy(workloads.bf16_bits(A).view(np.int16)).cuda().view(torch.bfloat16)
    need = fq.gemm_workspace_bytes_for(M, N, K, bits, g, act)
    assert 0 < need <= fq.gemm_noalloc_scratch_bytes(), f"case does not use the scratch: need {need}"
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    C_ref = torch.full((M, N), 3.0, dtype=tdt, device="cuda")
    C = torch.full((M, N), 7.0, dtype=tdt, device="cuda")
    st = fq.gemm_raw(Ad.data_ptr(), act, M, N, K, W_codes.data_ptr(), scales.data_ptr(), bits, g, C_ref.data_ptr(),
                     ws.data_ptr(), need, stream)
    assert st == fq.FQ_OK
    st = fq.gemm_noalloc_raw(Ad.data_ptr(), act, M, N, K, W_codes.data_ptr(), scales.data_ptr(), bits, g,
                             C.data_ptr(), stream)
    assert st == fq.FQ_OK, fq.status_string(st)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(C.float()).all())
    assert torch.equal(C.view(torch.int16), C_ref.view(torch.int16)), \
        f"fq_gemm_noalloc differs from fq_gemm: M={M} N={N} K={K} {dtype} [{fq.gemm_describe(M, N, K, bits, g)}]"


@pytest.mark.parametrize("K,N,bits,g,dtype,Ms", [
    (4096, 1024, 4, 128, "f16", (8, 3)),        # small-M kernel, K split over the grid
    (4096, 1024, 8, 0, "bf16", (16, 5)),
    (8192, 1024, 4, 64, "bf16", (40, 24)),      # tiled kernel, uniform split of K
    (1024, 8192, 4, 128, "bf16", (300, 260)),   # bf16 rows rewritten as binary16 (128-row blocks, N >= 8192)
])
def test_noalloc_matches_gemm_twice_second_smaller(K, N, bits, g, dtype, Ms):
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    W = workloads.weights_gaussian(K, N, seed=90 + bits, outlier_prob=1e-3)
    codes, scales = fq.quantize(torch.from_numpy(W).cuda(), bits, g)
    for i, M in enumerate(Ms):
        print(f"noalloc case K={K} N={N} int{bits} g={g or K} {dtype} M={M}: {fq.gemm_describe(M, N, K, bits, g)}",
              flush=True)
        _pair(fq, torch, codes, scales, K, N, bits, g, M, dtype, seed=100 + i)


def test_noalloc_captured_in_a_graph_replays_to_the_same_bits():
    """The callers the entry point is for: captured in a HIP graph (nothing is allocated and only kernels are
    enqueued, so the capture succeeds), replayed three times with eager work and synchronisations between the
    replays, each replay compared with fq_gemm's result."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N, bits, g = 4096, 1024, 4, 128
    W = workloads.weights_gaussian(K, N, seed=97, outlier_prob=1e-3)
    codes, scales = fq.quantize(torch.from_numpy(W).cuda(), bits, g)
    cases = []
    for M, dtype in ((8, "f16"), (40, "bf16")):
        A = workloads.activations(M, K, dtype, 120 + M)
        if dtype == "f16":
            Ad = torch.from_numpy(A).cuda()
        else:
            Ad = torch.from_numpy(workloads.bf16_bits(A).view(np.int16)).cuda().view(torch.bfloat16)
        act = fq.FQ_F16 if dtype == "f16" else fq.FQ_BF16
        assert 0 < fq.gemm_workspace_bytes_for(M, N, K, bits, g, act) <= fq.gemm_noalloc_scratch_bytes()
        ref = fq.gemm(Ad, codes, scales, bits, g)
        C = torch.empty_like(ref)
        # one eager call first: the library looks its scratch up on the first call on a device
        stream = torch.cuda.current_stream().cuda_stream
        assert fq.gemm_noalloc_raw(Ad.data_ptr(), act, M, N, K, codes.data_ptr(), scales.data_ptr(), bits, g,
                                   C.data_ptr(), stream) == fq.FQ_OK
        cases.append((Ad, act, M, ref, C))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stream = torch.cuda.current_stream().cuda_stream
        for Ad, act, M, ref, C in cases:
            st = fq.gemm_noalloc_raw(Ad.data_ptr(), act, M, N, K, codes.data_ptr(), scales.data_ptr(), bits, g,
                                     C.data_ptr(), stream)
            assert st == fq.FQ_OK, fq.status_string(st)
    for replay in range(3):
        for _, _, _, _, C in cases:
            C.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for _, _, M, ref, C in cases:
            assert torch.equal(C.view(torch.int16), ref.view(torch.int16)), f"replay {replay}, M={M}"
        again = fq.gemm(cases[0][0], codes, scales, bits, g)      # eager work between the replays
        assert torch.equal(again, cases[0][3])


def test_noalloc_rejects_what_does_not_fit_and_bad_arguments():
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N, M = 49152, 12288, 2048            # bf16 rows rewritten as binary16: 192 MiB of scratch
    assert fq.gemm_workspace_bytes_for(M, N, K, 4, 128, fq.FQ_BF16) > fq.gemm_noalloc_scratch_bytes()
    x = torch.zeros(64, dtype=torch.uint8, device="cuda")
    p = x.data_ptr()
    assert fq.gemm_noalloc_raw(p, fq.FQ_BF16, M, N, K, p, p, 4, 128, p, 0) == fq.FQ_ERR_WORKSPACE
    # a K-split last round (QKV-wide, 384 rows): its partial tiles exceed the scratch
    assert "tail=0x" not in fq.gemm_describe(384, 36864, 4096, 4, 128)
    assert fq.gemm_noalloc_raw(p, fq.FQ_F16, 384, 36864, 4096, p, p, 4, 128, p, 0) == fq.FQ_ERR_WORKSPACE
    assert fq.gemm_noalloc_raw(p, fq.FQ_F16, 8, 1024, 4096, p, p, 5, 128, p, 0) == fq.FQ_ERR_INVALID_ARG
    assert fq.gemm_noalloc_raw(None, fq.FQ_F16, 8, 1024, 4096, p, p, 4, 128, p, 0) == fq.FQ_ERR_INVALID_ARG
    assert fq.gemm_noalloc_raw(p, fq.FQ_F16, 0, 1024, 4096, p, p, 4, 128, p, 0) == fq.FQ_OK
