"""GPU parity at the full sizes of the benchmark configurations, on sampled output columns.

The oracle cannot multiply a 12288 x 49152 matrix in seconds, but every output column depends only on
its own weight column, so a sample of columns is quantised and multiplied by the oracle one by one
and compared with the same columns of the GPU result, which is computed on the whole matrix in the
launch configuration bench.py times.  Codes and scales of the sampled columns must match bit for bit.
"""
import numpy as np
import pytest

import oracle
from paper_2308_09723_amd import workloads

from gpu_util import TOL, from_dev_act, to_dev_act, torch_mod

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _sample_columns(N, count, seed):
    rng = np.random.default_rng(seed)
    cols = set(rng.integers(0, N, size=count).tolist())
    cols.update([0, 1, 15, 16, N - 17, N - 16, N - 1])          # first / last tiles
    return np.array(sorted(cols), dtype=np.int64)


def _structured_columns(N, seed, block=384, tile=16, extra=16):
    """A column sample that follows the kernels' tiling instead of chance.  The tiled kernel's blocks span
    384 columns (8 waves x 3 tiles of 16; 192 for its 4-wave shapes) and walk panels of four column blocks;
    the small-M kernel's blocks take runs of 1 - 36 tiles.  The sample holds
      * one column of EVERY 384-column block, its tile position (0..23) and its column inside the tile
        (0..15) advancing from block to block, so that every column block of every panel (hence every block
        of the grid, the K-split ones of a partly filled last round included) has a compared column;
      * every one of the 24 tile positions of the first, the middle and the last column block, plus the
        first and last column of each of these blocks;
      * the first and last tiles' edge columns and `extra` seeded random columns."""
    rng = np.random.default_rng(seed)
    nblk = -(-N // block)
    tpb = block // tile
    cols = set()
    for b in range(nblk):
        c = b * block + ((7 * b + 3) % tpb) * tile + (5 * b + 1) % tile
        cols.add(min(c, N - 1))
    for b in sorted({0, nblk // 2, nblk - 1}):
        lo, hi = b * block, min(N, (b + 1) * block)
        cols.update([lo, hi - 1])
        for t in range(tpb):
            c = lo + t * tile + (3 * t + b) % tile
            if c < hi:
                cols.add(c)
    cols.update([0, 1, 15, 16, N - 17, N - 16, N - 1])
    cols.update(rng.integers(0, N, size=extra).tolist())
    return np.array(sorted(cols), dtype=np.int64)


def _check_layer(W, bits, g, cases, cols, tag, sfmt="f16"):
    """cases: list of (M, dtype, seed).  Quantises W on the GPU, checks sampled columns against the oracle.
    sfmt: storage format of the scales ("f16", or "bf16" with bf16 activations)."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    K, N = W.shape
    Wd = torch.from_numpy(W).cuda()
    codes, scales = fq.quantize(Wd, bits, g, fq.FQ_SCALE_BF16 if sfmt == "bf16" else fq.FQ_SCALE_F16)
    del Wd
    cols_d = torch.from_numpy(cols).cuda()
    q_gpu = fq.unpack(codes, K, N, bits).index_select(1, cols_d).cpu().numpy()
    s_gpu = scales.index_select(1, cols_d).view(torch.int16).cpu().numpy().view(np.uint16)
    q_ref, s_ref = oracle.quantize(np.ascontiguousarray(W[:, cols]), bits, g, sfmt)
    s_ref_bits = oracle.bf16_scale_bits(s_ref) if sfmt == "bf16" else s_ref.view(np.uint16)
    assert np.array_equal(s_gpu, s_ref_bits), f"{tag}: scales differ on sampled columns"
    assert np.array_equal(q_gpu, q_ref), f"{tag}: codes differ on sampled columns"
    for M, dtype, seed in cases:
        A = workloads.activations(M, K, dtype, seed)
        C = fq.gemm(to_dev_act(A, dtype), codes, scales, bits, g)
        assert bool(torch.isfinite(C.float()).all()), f"{tag} M={M}: non-finite output"
        C_s = from_dev_act(C.index_select(1, cols_d), dtype)
        C_ref = oracle.gemm_ref(A, q_ref, s_ref)
        scale = np.max(np.abs(C_ref))
        err = np.max(np.abs(C_s - C_ref))
        _say(f"  {tag} int{bits} g={g or K} {dtype} M={M}: rel err {err / scale:.2e}  [{fq.gemm_describe(M, N, K, bits, g)}]")
        assert err <= TOL[dtype] * scale, f"{tag} M={M} {dtype}: {err} > {TOL[dtype]} * {scale}"


@pytest.mark.parametrize("layer", ["out_proj", "fc2", "qkv", "fc1"])
def test_opt175b_decode_layers_full_size(layer):
    """BASELINE configs[1]: int4, group 128, fp16, M = 1 and M = 8 — the shapes and plans bench.py times."""
    _say(f"full-size decode layer {layer}: generating weights")
    W = workloads.opt175b_weight(layer, seed=3)
    cols = _sample_columns(W.shape[1], 40, seed=11)
    _check_layer(W, 4, 128, [(1, "f16", 21), (8, "f16", 22)], cols, layer)


def test_opt175b_prefill_full_size_bf16():
    """BASELINE configs[2]: bf16 activations, M in {32, 128, 512, 2048}; int4 at the group size the
    heuristic picks from {256, 128, 64}, and int8 per column, on the out-proj shape."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    _say("full-size prefill: generating weights")
    W = workloads.opt175b_weight("out_proj", seed=4)
    cols = _sample_columns(W.shape[1], 24, seed=12)
    g_pick = fq.choose_group(torch.from_numpy(W).cuda(), 256, 64, 0.9)
    g_ref = oracle.choose_group(W, 256, 64, 0.9)
    _say(f"  heuristic picked g={g_pick} (oracle {g_ref})")
    assert g_pick == g_ref
    cases = [(32, "bf16", 31), (128, "bf16", 32), (512, "bf16", 33), (2048, "bf16", 34)]
    _check_layer(W, 4, g_pick, cases, cols, "out_proj")
    _check_layer(W, 8, 0, cases[1:3], cols, "out_proj")
    _check_layer(W, 4, 256 if g_pick != 256 else 128, [(512, "bf16", 35)], cols, "out_proj")
    # the 32- and 64-row blocks in their post-scaled form (one scale row per k-block), both activation types
    _check_layer(W, 4, 128, [(32, "f16", 36), (64, "f16", 37), (32, "bf16", 38), (64, "bf16", 39)], cols, "out_proj")


@pytest.mark.parametrize("layer", ["qkv", "fc1", "fc2", "out_proj"])
def test_opt175b_layers_full_size_structured_sample(layer):
    """BASELINE configs[1] and configs[2] on every layer shape, in the plans bench.py times, compared with the
    oracle on the structured column sample (every column block, every tile position): decode M = 1 and 8
    (fp16), prefill M = 512 and 2048 in bf16 AND fp16; FC2 (384 k-blocks to accumulate) also at M = 32 and
    128; QKV also with 8-bit codes, one group per column, at M = 2048."""
    _say(f"full-size layer {layer}: generating weights")
    W = workloads.opt175b_weight(layer, seed=7)
    cols = _structured_columns(W.shape[1], seed=17)
    _say(f"  {len(cols)} sampled columns of {W.shape[1]}")
    cases = [(1, "f16", 71), (8, "f16", 72), (512, "bf16", 73), (2048, "bf16", 74), (2048, "f16", 75)]
    if layer == "fc2":
        cases += [(32, "bf16", 76), (128, "bf16", 77), (128, "f16", 78)]
    _check_layer(W, 4, 128, cases, cols, layer)
    if layer == "qkv":
        _check_layer(W, 8, 0, [(2048, "bf16", 79), (2048, "f16", 80)], cols, layer)
        # bfloat16 scales (the scales of the activation's type): small-M, 32-row and 128-row kernels
        _check_layer(W, 4, 128, [(8, "bf16", 83), (32, "bf16", 84), (2048, "bf16", 85)], cols, layer + "-bf16scales", sfmt="bf16")


def test_out_proj_decode_every_column():
    """The out-proj layer (the one whose k-workers run the fewest iterations and whose K is split over the
    grid) at M = 1 and M = 8: codes, scales and the product compared with the oracle on ALL 12288 columns."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    _say("out-proj, every column: generating weights")
    W = workloads.opt175b_weight("out_proj", seed=8)
    K, N = W.shape
    codes, scales = fq.quantize(torch.from_numpy(W).cuda(), 4, 128)
    q_ref, s_ref = oracle.quantize(W, 4, 128)
    assert np.array_equal(scales.view(torch.int16).cpu().numpy().view(np.uint16), s_ref.view(np.uint16))
    assert np.array_equal(fq.unpack(codes, K, N, 4).cpu().numpy(), q_ref)
    for M, seed in ((1, 81), (8, 82)):
        A = workloads.activations(M, K, "f16", seed)
        C = from_dev_act(fq.gemm(to_dev_act(A, "f16"), codes, scales, 4, 128), "f16")
        C_ref = oracle.gemm_ref(A, q_ref, s_ref)
        scale = np.max(np.abs(C_ref))
        err = np.max(np.abs(C - C_ref))
        _say(f"  out_proj all columns M={M}: rel err {err / scale:.2e}  [{fq.gemm_describe(M, N, K, 4, 128)}]")
        assert err <= TOL["f16"] * scale


def test_heavy_tailed_stress_layer_full_size():
    """BASELINE configs[4]: K = 8192, N = 28672, Student-t weights, 1 % of columns x50; bf16 output."""
    _say("stress layer: generating weights")
    K, N = workloads.STRESS_LAYER
    W = workloads.weights_heavy_tail(K, N, seed=9)
    cols = _sample_columns(N, 24, seed=13)
    for bits in (4, 8):
        for g in (32, 128, 0):
            _check_layer(W, bits, g, [(1, "bf16", 41), (16, "bf16", 42), (256, "bf16", 43)], cols, "stress")


def test_moe_grouped_full_shapes():
    """BASELINE configs[3] shapes (d_model 4096, d_ff 16384, int4 g = 64, fp16), Zipf(1.1) top-2 routing of
    2048 tokens; 8 experts are materialised on the host (one forced empty) instead of 64."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    E = 8
    d_model, d_ff = workloads.MOE["d_model"], workloads.MOE["d_ff"]
    offsets, _ = workloads.zipf_routing(2048, E - 1, 2, 1.1, seed=5)
    offsets = np.concatenate([offsets[:4], [offsets[3]], offsets[4:]]).astype(np.int32)   # expert 3 gets no rows
    assert offsets[4] == offsets[3] and len(offsets) == E + 1
    rows = int(offsets[-1])
    _say(f"moe: rows per expert {np.diff(offsets).tolist()}")
    for (K, N, tag) in ((d_model, d_ff, "fc1"), (d_ff, d_model, "fc2")):
        A = workloads.activations(rows, K, "f16", 51)
        cols = _sample_columns(N, 12, seed=14)
        cols_d = torch.from_numpy(cols).cuda()
        codes_l, scales_l, qs, ss = [], [], [], []
        for e in range(E):
            W = workloads.weights_gaussian(K, N, 600 + e)
            c, s = fq.quantize(torch.from_numpy(W).cuda(), 4, 64)
            codes_l.append(c)
            scales_l.append(s.reshape(-1))
            q_ref, s_ref = oracle.quantize(np.ascontiguousarray(W[:, cols]), 4, 64)
            q_gpu = fq.unpack(c, K, N, 4).index_select(1, cols_d).cpu().numpy()
            assert np.array_equal(q_gpu, q_ref), f"moe {tag} expert {e}: codes differ"
            qs.append(q_ref)
            ss.append(s_ref)
        codes = torch.cat(codes_l)
        scales = torch.cat(scales_l)
        out = torch.full((rows, N), 5.0, dtype=torch.float16, device="cuda")
        fq.gemm_grouped(to_dev_act(A, "f16"), offsets.tolist(), codes, scales, 4, 64, N, out=out)
        C = out.index_select(1, cols_d).cpu().numpy().astype(np.float64)
        C_ref = oracle.gemm_ref_grouped(A, offsets, qs, ss)
        scale = np.max(np.abs(C_ref))
        err = np.max(np.abs(C - C_ref))
        _say(f"  moe {tag}: rel err {err / scale:.2e}")
        assert err <= TOL["f16"] * scale


def test_moe_grouped_all_64_experts():
    """BASELINE configs[3] with the routing bench.py times: all 64 experts' offsets (Zipf(1.1), top-2, 2048
    tokens, seed 5) plus the same routing with two experts emptied.  The 64 weight slots cycle through 8
    distinct matrices (host time); every expert index, offset and stride of the real launch is exercised."""
    from paper_2308_09723_amd import fq
    torch = torch_mod()
    E, D = workloads.MOE["experts"], 8
    d_model, d_ff = workloads.MOE["d_model"], workloads.MOE["d_ff"]
    offsets, _ = workloads.zipf_routing(2048, E, 2, 1.1, seed=5)
    counts = np.diff(offsets)
    counts2 = counts.copy()
    counts2[[2, 40]] = 0                                      # a popular and a rare expert without rows
    offsets2 = np.concatenate([[0], np.cumsum(counts2)]).astype(np.int32)
    _say(f"moe-64: rows per expert {counts.tolist()}")
    for (K, N, tag) in ((d_model, d_ff, "fc1"), (d_ff, d_model, "fc2")):
        cols = _structured_columns(N, seed=18, extra=4)
        cols_d = torch.from_numpy(cols).cuda()
        codes_l, scales_l, qs, ss = [], [], [], []
        for d in range(D):
            W = workloads.weights_gaussian(K, N, 700 + d)
            c, s = fq.quantize(torch.from_numpy(W).cuda(), 4, 64)
            codes_l.append(c)
            scales_l.append(s.reshape(-1))
            q_ref, s_ref = oracle.quantize(np.ascontiguousarray(W[:, cols]), 4, 64)
            assert np.array_equal(fq.unpack(c, K, N, 4).index_select(1, cols_d).cpu().numpy(), q_ref)
            qs.append(q_ref)
            ss.append(s_ref)
        codes = torch.cat([codes_l[e % D] for e in range(E)])
        scales = torch.cat([scales_l[e % D] for e in range(E)])
        del codes_l, scales_l
        for offs in (offsets, offsets2):
            rows = int(offs[-1])
            A = workloads.activations(rows, K, "f16", 52)
            out = torch.full((rows, N), 5.0, dtype=torch.float16, device="cuda")
            fq.gemm_grouped(to_dev_act(A, "f16"), offs.tolist(), codes, scales, 4, 64, N, out=out)
            assert bool(torch.isfinite(out.float()).all())
            C = out.index_select(1, cols_d).cpu().numpy().astype(np.float64)
            C_ref = oracle.gemm_ref_grouped(A, offs, [qs[e % D] for e in range(E)], [ss[e % D] for e in range(E)])
            scale = np.max(np.abs(C_ref))
            err = np.max(np.abs(C - C_ref))
            _say(f"  moe-64 {tag} rows={rows}: rel err {err / scale:.2e}")
            assert err <= TOL["f16"] * scale
        del codes, scales


@pytest.mark.parametrize("bits,g,K", [(4, 128, 4096), (4, 64, 3072), (8, 0, 4096)])
def test_split_tail_round_on_sampled_columns(bits, g, K):
    """QKV-wide products whose output tiles exceed the block slots by a partly filled last round: the plan
    splits those last tiles along K (checked through the plan's description) and a tail reduction adds
    their partial tiles.  Columns are sampled from every part of N, the last column blocks included."""
    from paper_2308_09723_amd import fq
    W = workloads.opt175b_weight("qkv", seed=6, rows=K)
    N = W.shape[1]
    cases = [(384, "bf16", 61), (768, "f16", 62), (1100, "bf16", 63)]     # 1100 rows: ragged last row block
    for M, _, _ in cases:
        desc = fq.gemm_describe(M, N, K, bits, g)
        _say(f"  M={M}: {desc}")
        assert "tail=0x" not in desc, desc
    # every column block has a compared column (all rows are compared), so every K-split tile is covered
    cols = _structured_columns(N, seed=15)
    extra = np.arange(N - 1536, N, 97)                       # denser over the last column blocks
    cols = np.array(sorted(set(cols.tolist()) | set(extra.tolist())), dtype=np.int64)
    _check_layer(W, bits, g, cases, cols, "qkv-tail")
