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
    return sorted(set(re.findall(r"\b(fq_[a-z_]+)\s*\(", text)))


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
    assert fq.codes_bytes(1024, 1024, 3) == 0
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
    (dict(bits=3), fq.FQ_ERR_INVALID_ARG),
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
    st, g = fq.choose_group_raw(16, 1024, 1024, 64, 64, 0.5, None, 0)
    assert st == fq.FQ_OK and g == 64                     # nothing to halve: answered on the host
    assert fq.status_string(fq.FQ_ERR_WORKSPACE) == "FQ_ERR_WORKSPACE"
    assert fq.status_string(99) == "FQ_ERR_UNKNOWN"


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
    assert call(bits=3) == fq.FQ_ERR_INVALID_ARG
    assert call(g=96) == fq.FQ_ERR_INVALID_ARG
    assert call(N=1032) == fq.FQ_ERR_UNSUPPORTED
    assert call(ws=0) == fq.FQ_ERR_WORKSPACE
    assert call(wsb=64) == fq.FQ_ERR_WORKSPACE
