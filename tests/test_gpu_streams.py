"""GPU checks of how the entry points behave on streams other than the default one and when two host
threads call them at the same time: results must be bit-identical to those of a plain call (the kernels
add in a fixed order), also for the grouped product, whose launches fork onto two library-owned side
streams and join back (serialised across host threads inside the library).
"""
import threading

import numpy as np
import pytest

from paper_2308_09723_amd import workloads

from gpu_util import to_dev_act, torch_mod

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _setup(fq, torch, seed):
    """A few products that cover the small-M kernel, a split of K with workspace, the bf16 rows rewritten as
    binary16 (workspace) and the grouped product."""
    K, N, g = 1024, 9216, 128
    W = workloads.weights_gaussian(K, N, seed, outlier_prob=1e-3)
    codes, scales = fq.quantize(torch.from_numpy(W).cuda(), 4, g)
    acts = {(M, dt): to_dev_act(workloads.activations(M, K, dt, seed + M), dt)
            for M, dt in ((3, "f16"), (40, "f16"), (300, "bf16"))}
    rows = [70, 0, 33, 129, 5]
    offsets = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    Ag = to_dev_act(workloads.activations(int(offsets[-1]), K, "f16", seed + 7), "f16")
    Ng = 768
    cg, sg = [], []
    for e in range(len(rows)):
        c, s = fq.quantize(torch.from_numpy(workloads.weights_gaussian(K, Ng, seed + 20 + e)).cuda(), 4, g)
        cg.append(c)
        sg.append(s.reshape(-1))
    return dict(K=K, N=N, g=g, codes=codes, scales=scales, acts=acts, offsets=offsets.tolist(), Ag=Ag, Ng=Ng,
                cg=torch.cat(cg), sg=torch.cat(sg))


def _run_all(fq, d):
    out = [fq.gemm(A, d["codes"], d["scales"], 4, d["g"]) for A in d["acts"].values()]
    out.append(fq.gemm_grouped(d["Ag"], d["offsets"], d["cg"], d["sg"], 4, d["g"], d["Ng"]))
    return out


def test_products_on_a_side_stream_match_the_default_stream():
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    d = _setup(fq, torch, 4100)
    for (M, dt) in d["acts"]:
        _say(f"  M={M} {dt}: {fq.gemm_describe(M, d['N'], d['K'], 4, d['g'])}")
    ref = [t.clone() for t in _run_all(fq, d)]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            got = _run_all(fq, d)
    side.synchronize()
    for r, c in zip(ref, got):
        assert torch.equal(r, c)


def test_two_host_threads_on_their_own_streams():
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    data = [_setup(fq, torch, 4200), _setup(fq, torch, 4300)]
    refs = [[t.clone() for t in _run_all(fq, d)] for d in data]
    torch.cuda.synchronize()
    start = threading.Barrier(2)
    failures = []

    def worker(i):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                start.wait(timeout=60)
                for it in range(25):
                    got = _run_all(fq, data[i])
                    stream.synchronize()
                    for r, c in zip(refs[i], got):
                        if not torch.equal(r, c):
                            failures.append((i, it))
                            return
        except Exception as exc:      # noqa: BLE001 - reported below
            failures.append((i, repr(exc)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a worker did not finish"
    assert not failures, failures


def test_products_captured_in_a_graph_replay_to_the_same_bits():
    """fq_gemm enqueues kernels only (no memsets, no synchronisation, no allocation), so a caller may
    capture it in a HIP graph: three replays, with eager work and synchronisations between them, each
    compared with the eager result."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    d = _setup(fq, torch, 4400)
    acts = list(d["acts"].values())
    ref = [fq.gemm(A, d["codes"], d["scales"], 4, d["g"]).clone() for A in acts]
    outs = [torch.empty_like(r) for r in ref]
    ws = [torch.empty(max(16, fq.gemm_workspace_bytes(A.shape[0], d["N"], d["K"], 4, d["g"])), dtype=torch.uint8,
                      device="cuda") for A in acts]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for A, C, w in zip(acts, outs, ws):
            fq.gemm(A, d["codes"], d["scales"], 4, d["g"], out=C, workspace=w)
    for replay in range(3):
        for C in outs:
            C.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for r, c in zip(ref, outs):
            assert torch.equal(r, c), f"replay {replay}"
        # eager work between the replays
        again = fq.gemm(acts[0], d["codes"], d["scales"], 4, d["g"])
        assert torch.equal(again, ref[0])


def test_integer_path_captured_in_a_graph_replays_to_the_same_bits():
    """fq_quantize_act_i8 and fq_gemm_w4a8 enqueue kernels only as well: the activation quantiser and the products
    of the small-M kernel (with a split of K over the grid) and of the tiled kernel captured in one graph."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N, g = 2048, 1536, 128
    W = workloads.weights_gaussian(K, N, 4500, outlier_prob=1e-3)
    codes, z, t = fq.quantize_w4a8(torch.from_numpy(W).cuda(), g)
    cases = []
    for M in (6, 200):
        A = to_dev_act(workloads.activations(M, K, "f16", 4500 + M), "f16")
        Aq, alpha = fq.quantize_act_i8(A)
        ref = fq.gemm_w4a8(Aq, alpha, codes, z, t, g, torch.float16).clone()
        ws = torch.empty(max(16, fq.gemm_w4a8_workspace_bytes(M, N, K, g)), dtype=torch.uint8, device="cuda")
        cases.append((A, torch.empty_like(Aq), torch.empty_like(alpha), ws, ref, torch.empty_like(ref)))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stream = torch.cuda.current_stream().cuda_stream
        for A, Aq, alpha, ws, ref, C in cases:
            M = A.shape[0]
            assert fq.quantize_act_i8_raw(A.data_ptr(), fq.FQ_F16, M, K, Aq.data_ptr(), alpha.data_ptr(), stream) == fq.FQ_OK
            fq.gemm_w4a8(Aq, alpha, codes, z, t, g, torch.float16, out=C, workspace=ws)
    for replay in range(3):
        for _, Aq, _, _, _, C in cases:
            C.fill_(7.0)
            Aq.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for A, _, _, _, ref, C in cases:
            assert torch.equal(ref, C), f"replay {replay}, M={A.shape[0]}"


@pytest.mark.parametrize("nbytes", [16, 1 << 20, (1 << 22) + 4096 + 48, 256 * 768 * 16 * 4 + 16])
def test_stream_read_probe_reads_every_word_once(nbytes):
    """The measurement helper that bench.py times as the streaming-read ceiling: the XOR of its per-block
    checksum words equals the XOR of all 32-bit words of the buffer (every word read, none twice)."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    rng = np.random.default_rng(nbytes)
    host = rng.integers(0, 2 ** 32, size=nbytes // 4, dtype=np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).cuda()
    sink = torch.zeros(256, dtype=torch.int32, device="cuda")
    st = fq.stream_read_probe_raw(buf.data_ptr(), nbytes, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == fq.FQ_OK
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert got == np.bitwise_xor.reduce(host)
    assert fq.stream_read_probe_raw(buf.data_ptr(), 24, sink.data_ptr(), 0) == fq.FQ_ERR_INVALID_ARG
    assert fq.stream_read_probe_raw(None, 16, sink.data_ptr(), 0) == fq.FQ_ERR_INVALID_ARG


def test_mfma_rate_probe_counts_what_it_says():
    """The measurement helper that bench.py times as the matrix pipes' ceiling: with all operands 1 (binary16 1.0,
    or int8 1 for the integer instruction) every accumulator element grows by the MFMA's depth (32 or 64) per
    MFMA folded into it (4 k-steps x iterations), so each thread's checksum is known; buffers that are too small
    are refused."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    nb, sb = fq.mfma_rate_probe_operand_bytes(), fq.mfma_rate_probe_sink_bytes()
    ones16 = torch.ones(nb // 2, dtype=torch.float16, device="cuda")
    ones8 = torch.ones(nb, dtype=torch.int8, device="cuda")
    sink = torch.zeros(sb // 4, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    iters = 3
    for int8, ones, depth in ((0, ones16, 32), (1, ones8, 64)):
        for lds in (0, 1):
            sink.zero_()
            assert fq.mfma_rate_probe_raw(ones.data_ptr(), nb, sink.data_ptr(), sb, iters, lds, int8, stream) == fq.FQ_OK
            torch.cuda.synchronize()
            # 8 x 3 accumulator tiles, four elements each, every element = depth * 4 * iters
            want = 8 * 3 * 4 * float(depth) * 4 * iters
            assert bool((sink == want).all()), (int8, lds, float(sink.min()), float(sink.max()), want)
        assert fq.mfma_rate_probe_flops(iters, int8) == 1024 * 8 * iters * 96 * 2.0 * 16 * 16 * depth
    ones = ones16
    assert fq.mfma_rate_probe_raw(ones.data_ptr(), nb - 16, sink.data_ptr(), sb, iters, 0, 0, 0) == fq.FQ_ERR_WORKSPACE
    assert fq.mfma_rate_probe_raw(ones.data_ptr(), nb, sink.data_ptr(), sb - 4, iters, 0, 0, 0) == fq.FQ_ERR_WORKSPACE
    assert fq.mfma_rate_probe_raw(None, nb, sink.data_ptr(), sb, iters, 0, 0, 0) == fq.FQ_ERR_INVALID_ARG
    assert fq.mfma_rate_probe_raw(ones.data_ptr(), nb, sink.data_ptr(), sb, 0, 0, 0, 0) == fq.FQ_ERR_INVALID_ARG
