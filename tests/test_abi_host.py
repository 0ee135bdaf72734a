"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes follow their closed forms and invalid arguments are rejected before any launch."""
import os
import re

import pytest

from paper_2308_09723_amd import fq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "fq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = fq.load()
    declared = _declared_symbols()
    assert len(declared) >= 12
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(fq.EXPORTED) == declared
    assert fq.version().count(".") == 1


def test_size_queries():
    assert fq.codes_bytes(1024, 1024, 4) == 1024 * 1024 // 2
    assert fq.codes_bytes(1024, 1024, 8) == 1024 * 1024
    assert fq.codes_bytes(1024, 1024, 3) == 1024 * 1024 * 3 // 8
    assert fq.codes_bytes(1024, 1024, 5) == 0
    assert fq.scales_bytes(1024, 1024, 128) == 8 * 1024 * 2
    assert fq.scales_bytes(1024, 1024, 0) == 1024 * 2
    assert fq.scales_bytes(1024, 1024, 1024) == 1024 * 2
    assert fq.scales_bytes(1024, 1024, 100) == 0
    # bits per weight = b + 16 / g
    K, N, g = 12288, 12288, 64
    total_bits = 8 * (fq.codes_bytes(K, N, 4) + fq.scales_bytes(K, N, g))
    assert total_bits == K * N * 4 + (K * N // g) * 16
    assert fq.gemm_workspace_bytes(0, 1024, 1024, 4, 128) == 0
    assert fq.gemm_workspace_bytes(4, 1000, 1024, 4, 128) == 0     # invalid shape -> 0


@pytest.mark.parametrize("args,expect", [
    (dict(W=0), fq.FQ_ERR_INVALID_ARG),
    (dict(codes=0), fq.FQ_ERR_INVALID_ARG),
    (dict(scales=0), fq.FQ_ERR_INVALID_ARG),
    (dict(bits=5), fq.FQ_ERR_INVALID_ARG),
    (dict(bits=2), fq.FQ_ERR_INVALID_ARG),
    (dict(bits=16), fq.FQ_ERR_INVALID_ARG),
    (dict(g=100), fq.FQ_ERR_INVALID_ARG),          # does not divide K
    (dict(g=-1), fq.FQ_ERR_INVALID_ARG),
    (dict(g=2048), fq.FQ_ERR_INVALID_ARG),         # larger than K
    (dict(K=0), fq.FQ_ERR_INVALID_ARG),
    (dict(g=16), fq.FQ_ERR_UNSUPPORTED),           # divides K but below the 32-row minimum
    (dict(N=1000), fq.FQ_ERR_UNSUPPORTED),         # not a multiple of 16
    (dict(K=1088, g=0, bits=4), fq.FQ_ERR_UNSUPPORTED),   # not a multiple of 128
])
def test_quantize_rejects_bad_arguments_on_the_host(args, expect):
    a = dict(W=16, K=1024, N=1024, bits=4, g=128, codes=16, scales=16)
    a.update(args)
    st = fq.quantize_raw(a["W"] or None, a["K"], a["N"], a["bits"], a["g"], a["codes"] or None, a["scales"] or None)
    assert st == expect, fq.status_string(st)


def test_gemm_rejects_bad_arguments_on_the_host():
    ok = dict(A=16, act=fq.FQ_F16, M=4, N=1024, K=1024, codes=16, scales=16, bits=4, g=128, C=16, ws=16, wsb=1 << 30)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return fq.gemm_raw(a["A"] or None, a["act"], a["M"], a["N"], a["K"], a["codes"] or None, a["scales"] or None,
                           a["bits"], a["g"], a["C"] or None, a["ws"] or None, a["wsb"])

    assert call(A=0) == fq.FQ_ERR_INVALID_ARG
    assert call(C=0) == fq.FQ_ERR_INVALID_ARG
    assert call(act=7) == fq.FQ_ERR_INVALID_ARG
    assert call(M=-1) == fq.FQ_ERR_INVALID_ARG
    assert call(bits=5) == fq.FQ_ERR_INVALID_ARG
    assert call(g=96) == fq.FQ_ERR_INVALID_ARG             # 1024 % 96 != 0
    assert call(N=1032) == fq.FQ_ERR_UNSUPPORTED
    assert call(K=1056, g=0, bits=8) == fq.FQ_ERR_UNSUPPORTED
    assert call(M=0, A=0, C=0) == fq.FQ_OK                 # empty product is a no-op
    need = fq.gemm_workspace_bytes(4, 1024, 1024, 4, 128)
    if need:
        assert call(ws=0) == fq.FQ_ERR_WORKSPACE
        assert call(wsb=need - 1) == fq.FQ_ERR_WORKSPACE


def test_grouped_and_heuristic_argument_checks():
    st = fq.gemm_grouped_raw(16, fq.FQ_F16, [0, 4, 2], 1024, 1024, 16, 16, 4, 64, 16)
    assert st == fq.FQ_ERR_INVALID_ARG                    # offsets decrease
    st = fq.gemm_grouped_raw(16, fq.FQ_F16, [1, 4], 1024, 1024, 16, 16, 4, 64, 16)
    assert st == fq.FQ_ERR_INVALID_ARG                    # offsets[0] != 0
    st = fq.gemm_grouped_raw(None, fq.FQ_F16, [0, 0, 0], 1024, 1024, 16, 16, 4, 64, None)
    assert st == fq.FQ_OK                                 # no rows at all
    st, _ = fq.choose_group_raw(None, 1024, 1024, 0, 32, 0.5, 16, 1 << 30)
    assert st == fq.FQ_ERR_INVALID_ARG
    st, _ = fq.choose_group_raw(16, 1024, 1024, 0, 32, 1.5, 16, 1 << 30)
    assert st == fq.FQ_ERR_INVALID_ARG
    st, _ = fq.choose_group_raw(16, 1024, 1024, 100, 32, 0.5, 16, 1 << 30)
    assert st == fq.FQ_ERR_INVALID_ARG
    st, _ = fq.choose_group_raw(16, 1024, 1024, 0, 32, 0.5, None, 0)
    assert st == fq.FQ_ERR_WORKSPACE
    st, _ = fq.choose_group_raw(16, 1024, 1032, 0, 32, 0.5, 16, 1 << 30)
    assert st == fq.FQ_ERR_UNSUPPORTED                    # N must be a multiple of 16
    st, g = fq.choose_group_raw(16, 1024, 1024, 64, 64, 0.5, None, 0)
    assert st == fq.FQ_OK and g == 64                     # nothing to halve: answered on the host
    assert fq.status_string(fq.FQ_ERR_WORKSPACE) == "FQ_ERR_WORKSPACE"
    assert fq.status_string(99) == "FQ_ERR_UNKNOWN"


def test_scale_format_argument_checks():
    """The *_sf entry points: unknown formats are invalid, bf16 scales go with bf16 activations only, and
    the plain entry points are the binary16 format."""
    F16, BF16 = fq.FQ_SCALE_F16, fq.FQ_SCALE_BF16
    assert fq.quantize_sf_raw(16, 1024, 1024, 4, 128, 2, 16, 16) == fq.FQ_ERR_INVALID_ARG
    assert fq.quantize_sf_raw(16, 1024, 1024, 4, 128, -1, 16, 16) == fq.FQ_ERR_INVALID_ARG
    assert fq.quantize_sf_raw(None, 1024, 1024, 4, 128, BF16, 16, 16) == fq.FQ_ERR_INVALID_ARG
    assert fq.quantize_sf_raw(16, 1024, 1000, 4, 128, BF16, 16, 16) == fq.FQ_ERR_UNSUPPORTED

    def gemm(act, sf, **kw):
        a = dict(A=16, M=4, N=1024, K=1024, codes=16, scales=16, bits=4, g=128, C=16)
        a.update(kw)
        return fq.gemm_sf_raw(a["A"] or None, act, a["M"], a["N"], a["K"], a["codes"], a["scales"], sf, a["bits"],
                              a["g"], a["C"], 16, 1 << 30)

    assert gemm(fq.FQ_F16, BF16) == fq.FQ_ERR_UNSUPPORTED
    assert gemm(fq.FQ_F16, BF16, M=0) == fq.FQ_ERR_UNSUPPORTED        # refused whatever the size
    assert gemm(fq.FQ_BF16, 5) == fq.FQ_ERR_INVALID_ARG
    assert gemm(9, F16) == fq.FQ_ERR_INVALID_ARG
    assert gemm(fq.FQ_BF16, BF16, A=0) == fq.FQ_ERR_INVALID_ARG
    assert gemm(fq.FQ_BF16, BF16, M=0, A=0) == fq.FQ_OK
    assert gemm(fq.FQ_BF16, BF16, g=96) == fq.FQ_ERR_INVALID_ARG
    st = fq.gemm_grouped_sf_raw(16, fq.FQ_F16, [0, 4], 1024, 1024, 16, 16, BF16, 4, 64, 16)
    assert st == fq.FQ_ERR_UNSUPPORTED
    st = fq.gemm_grouped_sf_raw(16, fq.FQ_BF16, [0, 4, 2], 1024, 1024, 16, 16, BF16, 4, 64, 16)
    assert st == fq.FQ_ERR_INVALID_ARG
    st = fq.gemm_grouped_sf_raw(None, fq.FQ_BF16, [0, 0], 1024, 1024, 16, 16, BF16, 4, 64, None)
    assert st == fq.FQ_OK
    assert fq.quant_error_sf_raw(16, 1024, 1024, 4, 128, 3, 16, 16, 16, 1 << 20)[0] == fq.FQ_ERR_INVALID_ARG
    assert fq.quant_error_sf_raw(16, 1024, 1024, 4, 128, BF16, 16, 16, None, 0)[0] == fq.FQ_ERR_WORKSPACE


def test_quant_error_argument_checks():
    """Validation precedes every launch, so these calls never touch a GPU."""
    assert fq.quant_error_workspace_bytes(0, 16) == 0
    assert fq.quant_error_workspace_bytes(1024, 1024) == 16 + 16 * 4 * 16      # 4 column x 16 row blocks
    ok = dict(W=16, K=1024, N=1024, bits=4, g=128, codes=16, scales=16, ws=16, wsb=1 << 20)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return fq.quant_error_raw(a["W"] or None, a["K"], a["N"], a["bits"], a["g"], a["codes"] or None,
                                  a["scales"] or None, a["ws"] or None, a["wsb"])[0]

    assert call(W=0) == fq.FQ_ERR_INVALID_ARG
    assert call(codes=0) == fq.FQ_ERR_INVALID_ARG
    assert call(scales=0) == fq.FQ_ERR_INVALID_ARG
    assert call(bits=5) == fq.FQ_ERR_INVALID_ARG
    assert call(g=96) == fq.FQ_ERR_INVALID_ARG
    assert call(N=1032) == fq.FQ_ERR_UNSUPPORTED
    assert call(ws=0) == fq.FQ_ERR_WORKSPACE
    assert call(wsb=64) == fq.FQ_ERR_WORKSPACE


def test_plans_are_consistent_over_many_shapes():
    """The plan (host code) for a seeded sweep of shapes: its description parses, the split of K covers K,
    a split tail round concerns fewer tiles than there are, and the workspace query matches the number of
    binary32 partial copies the plan writes."""
    import re
    import numpy as np
    rng = np.random.default_rng(11)
    seen = set()
    for _ in range(600):
        bits = int(rng.choice([3, 4, 8]))
        kblk = 64 if bits == 8 else 128
        K = kblk * int(rng.integers(1, 400))
        N = 16 * int(rng.integers(1, 3200))
        M = int(rng.choice([1, 3, 8, 16, 17, 32, 33, 64, 65, 100, 128, 129, 256, 384, 512, 777, 1024, 2048, 4096]))
        gs = [g for g in (32, 64, 128, 256, 0) if g == 0 or K % g == 0]
        g = int(rng.choice(gs))
        desc = fq.gemm_describe(M, N, K, bits, g)
        ws = fq.gemm_workspace_bytes_for(M, N, K, bits, g, fq.FQ_F16)
        ws_bf16 = fq.gemm_workspace_bytes_for(M, N, K, bits, g, fq.FQ_BF16)
        assert fq.gemm_workspace_bytes(M, N, K, bits, g) == max(ws, ws_bf16)
        # bfloat16 scales take the same path as binary16 ones (rows rewritten as binary16 for wide matrices)
        assert fq.gemm_workspace_bytes_for(M, N, K, bits, g, fq.FQ_BF16, fq.FQ_SCALE_BF16) == ws_bf16
        KB = K // kblk
        if desc.startswith("small-m"):
            f = dict(re.findall(r"(\w+)=(\d+)", desc))
            seen.add("small")
            assert M <= 16
            assert 1 <= int(f["gp"]) * int(f["kw"]) == int(f["waves"]) <= 12
            assert int(f["au"]) in (1, 2, 4) and M * (kblk // 8) <= int(f["au"]) * 64 * int(f["gp"])
            splits = int(f["splits"])
            assert 1 <= splits <= 8
            assert ws == (splits * M * N * 4 if splits > 1 else 0)
        else:
            m = re.match(r"tiled mt=(\d+) waves=(\d+) splits=(\d+) kb_per_split=(\d+) tail=(\d+)x(\d+)", desc)
            assert m, desc
            mt, waves, splits, kbs, tail_tiles, tail_splits = map(int, m.groups())
            seen.add("tail" if tail_tiles else ("split" if splits > 1 else "tiled"))
            assert M > 16 and mt in (2, 4, 8) and waves in (4, 8)
            assert mt == 8 or M <= 256                     # the small block shapes compete up to 256 rows only
            assert mt == 2 or mt * 8 < M                   # no block more than twice as tall as the matrix
            # k-blocks of the block shape: 8-bit codes in the 128-row, 8-wave shape go two 64-row layout
            # blocks at a time when a k-block of 128 rows stays inside one scale group
            if bits == 8 and mt == 8 and waves == 8 and K % 128 == 0 and (g or K) % 128 == 0:
                KB = K // 128
                seen.add("wide")
            assert splits >= 1 and kbs * splits >= KB and kbs * (splits - 1) < KB
            # bf16 rows are rewritten as binary16 for the 128-row shapes of wide matrices
            # (the rewritten rows, M row scales, the scale matrix's two powers of two and 256 words of their search)
            extra = (-(-(M * K * 2) // 256) * 256 + (M + 2 + 256) * 4) if (mt == 8 and N >= 8192) else 0
            assert ws_bf16 == ws + extra
            tiles = -(-(N // 16) // (waves * 3)) * -(-M // (mt * 16))
            if tail_tiles:
                assert splits == 1 and 0 < tail_tiles < tiles and 2 <= tail_splits <= 8
                assert ws == tail_splits * M * N * 4
            else:
                assert ws == (splits * M * N * 4 if splits > 1 else 0)
    assert {"small", "tiled", "split", "tail", "wide"} <= seen, seen
