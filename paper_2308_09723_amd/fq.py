"""ctypes binding of libfq (argument marshalling only).

Function names and arguments mirror ``include/fq.h``.  The ``*_raw`` functions
take integer device addresses exactly as the C ABI does; the helpers below them
take torch tensors (torch is used for device memory and streams only).
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfq.so")

FQ_OK = 0
FQ_ERR_INVALID_ARG = 1
FQ_ERR_UNSUPPORTED = 2
FQ_ERR_WORKSPACE = 3
FQ_ERR_HIP = 4
FQ_F16 = 0
FQ_BF16 = 1
FQ_SCALE_F16 = 0
FQ_SCALE_BF16 = 1

_lib = None


class FqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


def load(build_if_missing: bool = True) -> ctypes.CDLL:
    """Loads libfq.so (building it with hipcc first if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build

        build.build_lib(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, vp, sz, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
    sigs = {
        "fq_codes_bytes": (sz, [i64, i64, i32]),
        "fq_scales_bytes": (sz, [i64, i64, i32]),
        "fq_gemm_workspace_bytes": (sz, [i64, i64, i64, i32, i32]),
        "fq_gemm_workspace_bytes_for": (sz, [i64, i64, i64, i32, i32, i32, i32]),
        "fq_gemm_grouped_workspace_bytes": (sz, [i64, i32, i64, i64, i32, i32]),
        "fq_choose_group_workspace_bytes": (sz, [i64, i64, i32, i32]),
        "fq_quantize": (i32, [vp, i64, i64, i32, i32, vp, vp, vp]),
        "fq_unpack": (i32, [vp, i64, i64, i32, vp, vp]),
        "fq_choose_group": (i32, [vp, i64, i64, i32, i32, f32, ctypes.POINTER(ctypes.c_int), vp, sz, vp]),
        "fq_quant_error_workspace_bytes": (sz, [i64, i64]),
        "fq_quant_error": (i32, [vp, i64, i64, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double),
                                 ctypes.POINTER(ctypes.c_double), vp, sz, vp]),
        "fq_gemm": (i32, [vp, i32, i64, i64, i64, vp, vp, i32, i32, vp, vp, sz, vp]),
        "fq_gemm_grouped": (i32, [vp, i32, ctypes.POINTER(ctypes.c_int32), i32, i64, i64, vp, vp, i32, i32,
                                  vp, vp, sz, vp]),
        "fq_quantize_sf": (i32, [vp, i64, i64, i32, i32, i32, vp, vp, vp]),
        "fq_quant_error_sf": (i32, [vp, i64, i64, i32, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double),
                                    ctypes.POINTER(ctypes.c_double), vp, sz, vp]),
        "fq_gemm_sf": (i32, [vp, i32, i64, i64, i64, vp, vp, i32, i32, i32, vp, vp, sz, vp]),
        "fq_gemm_grouped_sf": (i32, [vp, i32, ctypes.POINTER(ctypes.c_int32), i32, i64, i64, vp, vp, i32, i32, i32,
                                     vp, vp, sz, vp]),
        "fq_gemm_noalloc": (i32, [vp, i32, i64, i64, i64, vp, vp, i32, i32, vp, vp]),
        "fq_gemm_noalloc_scratch_bytes": (sz, []),
        "fq_zscale_bytes": (sz, [i64, i64, i32]),
        "fq_quantize_w4a8": (i32, [vp, i64, i64, i32, vp, vp, vp, vp]),
        "fq_quantize_act_i8": (i32, [vp, i32, i64, i64, vp, vp, vp]),
        "fq_unpack_w4a8": (i32, [vp, i64, i64, vp, vp]),
        "fq_gemm_w4a8_workspace_bytes": (sz, [i64, i64, i64, i32]),
        "fq_gemm_w4a8": (i32, [vp, vp, i64, i64, i64, vp, vp, vp, i32, vp, i32, vp, sz, vp]),
        "fq_gemm_describe": (i32, [i64, i64, i64, i32, i32, ctypes.c_char_p, sz]),
        "fq_stream_read_probe": (i32, [vp, sz, vp, vp]),
        "fq_mfma_rate_probe_operand_bytes": (sz, []),
        "fq_mfma_rate_probe_sink_bytes": (sz, []),
        "fq_mfma_rate_probe_flops": (ctypes.c_double, [i32, i32]),
        "fq_mfma_rate_probe": (i32, [vp, sz, vp, sz, i32, i32, i32, vp]),
        "fq_status_string": (ctypes.c_char_p, [i32]),
        "fq_version": (ctypes.c_char_p, []),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


EXPORTED = [
    "fq_codes_bytes", "fq_scales_bytes", "fq_gemm_workspace_bytes", "fq_gemm_grouped_workspace_bytes",
    "fq_choose_group_workspace_bytes", "fq_quantize", "fq_unpack", "fq_choose_group", "fq_gemm",
    "fq_gemm_grouped", "fq_gemm_describe", "fq_status_string", "fq_version",
    "fq_quant_error_workspace_bytes", "fq_quant_error",
    "fq_quantize_sf", "fq_quant_error_sf", "fq_gemm_sf", "fq_gemm_grouped_sf", "fq_gemm_workspace_bytes_for",
    "fq_stream_read_probe", "fq_gemm_noalloc", "fq_gemm_noalloc_scratch_bytes",
    "fq_mfma_rate_probe_operand_bytes", "fq_mfma_rate_probe_sink_bytes", "fq_mfma_rate_probe_flops", "fq_mfma_rate_probe",
    "fq_zscale_bytes", "fq_unpack_w4a8", "fq_quantize_w4a8", "fq_quantize_act_i8", "fq_gemm_w4a8_workspace_bytes", "fq_gemm_w4a8",
]


def stream_read_probe_raw(buf_ptr, nbytes, sink_ptr, stream=0):
    return int(load().fq_stream_read_probe(buf_ptr, nbytes, sink_ptr, stream))


def mfma_rate_probe_operand_bytes():
    return int(load().fq_mfma_rate_probe_operand_bytes())


def mfma_rate_probe_sink_bytes():
    return int(load().fq_mfma_rate_probe_sink_bytes())


def mfma_rate_probe_flops(iterations, int8=0):
    return float(load().fq_mfma_rate_probe_flops(int(iterations), int(int8)))


def mfma_rate_probe_raw(operands_ptr, operand_bytes, sink_ptr, sink_bytes, iterations, lds_reads, int8=0, stream=0):
    return int(load().fq_mfma_rate_probe(operands_ptr, operand_bytes, sink_ptr, sink_bytes, iterations, lds_reads,
                                         int8, stream))


def status_string(status: int) -> str:
    return load().fq_status_string(int(status)).decode()


def version() -> str:
    return load().fq_version().decode()


# ------------------------------------------------------------------ raw (addresses) layer
def codes_bytes(K, N, bits):
    return int(load().fq_codes_bytes(K, N, bits))


def scales_bytes(K, N, group_size):
    return int(load().fq_scales_bytes(K, N, group_size))


def gemm_workspace_bytes(M, N, K, bits, group_size):
    return int(load().fq_gemm_workspace_bytes(M, N, K, bits, group_size))


def gemm_workspace_bytes_for(M, N, K, bits, group_size, act_dtype, scale_format=FQ_SCALE_F16):
    return int(load().fq_gemm_workspace_bytes_for(M, N, K, bits, group_size, act_dtype, scale_format))


def gemm_describe(M, N, K, bits, group_size):
    buf = ctypes.create_string_buffer(256)
    st = int(load().fq_gemm_describe(M, N, K, bits, group_size, buf, 256))
    if st != FQ_OK:
        raise FqError(st, "fq_gemm_describe")
    return buf.value.decode()


def choose_group_workspace_bytes(K, N, g_start, g_min):
    return int(load().fq_choose_group_workspace_bytes(K, N, g_start, g_min))


def quantize_raw(W_ptr, K, N, bits, group_size, codes_ptr, scales_ptr, stream=0):
    return int(load().fq_quantize(W_ptr, K, N, bits, group_size, codes_ptr, scales_ptr, stream))


def quantize_sf_raw(W_ptr, K, N, bits, group_size, scale_format, codes_ptr, scales_ptr, stream=0):
    return int(load().fq_quantize_sf(W_ptr, K, N, bits, group_size, scale_format, codes_ptr, scales_ptr, stream))


def unpack_raw(codes_ptr, K, N, bits, q_ptr, stream=0):
    return int(load().fq_unpack(codes_ptr, K, N, bits, q_ptr, stream))


def choose_group_raw(W_ptr, K, N, g_start, g_min, alpha, ws_ptr, ws_bytes, stream=0):
    out = ctypes.c_int(-1)
    st = int(load().fq_choose_group(W_ptr, K, N, g_start, g_min, alpha, ctypes.byref(out), ws_ptr, ws_bytes,
                                    stream))
    return st, out.value


def quant_error_workspace_bytes(K, N):
    return int(load().fq_quant_error_workspace_bytes(K, N))


def quant_error_raw(W_ptr, K, N, bits, group_size, codes_ptr, scales_ptr, ws_ptr, ws_bytes, stream=0):
    sse = ctypes.c_double(-1.0)
    mx = ctypes.c_double(-1.0)
    st = int(load().fq_quant_error(W_ptr, K, N, bits, group_size, codes_ptr, scales_ptr, ctypes.byref(sse),
                                   ctypes.byref(mx), ws_ptr, ws_bytes, stream))
    return st, sse.value, mx.value


def quant_error_sf_raw(W_ptr, K, N, bits, group_size, scale_format, codes_ptr, scales_ptr, ws_ptr, ws_bytes,
                       stream=0):
    sse = ctypes.c_double(-1.0)
    mx = ctypes.c_double(-1.0)
    st = int(load().fq_quant_error_sf(W_ptr, K, N, bits, group_size, scale_format, codes_ptr, scales_ptr,
                                      ctypes.byref(sse), ctypes.byref(mx), ws_ptr, ws_bytes, stream))
    return st, sse.value, mx.value


def gemm_raw(A_ptr, act_dtype, M, N, K, codes_ptr, scales_ptr, bits, group_size, C_ptr, ws_ptr, ws_bytes,
             stream=0):
    return int(load().fq_gemm(A_ptr, act_dtype, M, N, K, codes_ptr, scales_ptr, bits, group_size, C_ptr,
                              ws_ptr, ws_bytes, stream))


def gemm_noalloc_raw(A_ptr, act_dtype, M, N, K, codes_ptr, scales_ptr, bits, group_size, C_ptr, stream=0):
    return int(load().fq_gemm_noalloc(A_ptr, act_dtype, M, N, K, codes_ptr, scales_ptr, bits, group_size, C_ptr,
                                      stream))


def gemm_noalloc_scratch_bytes():
    return int(load().fq_gemm_noalloc_scratch_bytes())


def gemm_sf_raw(A_ptr, act_dtype, M, N, K, codes_ptr, scales_ptr, scale_format, bits, group_size, C_ptr, ws_ptr,
                ws_bytes, stream=0):
    return int(load().fq_gemm_sf(A_ptr, act_dtype, M, N, K, codes_ptr, scales_ptr, scale_format, bits, group_size,
                                 C_ptr, ws_ptr, ws_bytes, stream))


def gemm_grouped_raw(A_ptr, act_dtype, offsets, N, K, codes_ptr, scales_ptr, bits, group_size, C_ptr,
                     ws_ptr=None, ws_bytes=0, stream=0):
    E = len(offsets) - 1
    arr = (ctypes.c_int32 * (E + 1))(*[int(o) for o in offsets])
    return int(load().fq_gemm_grouped(A_ptr, act_dtype, arr, E, N, K, codes_ptr, scales_ptr, bits, group_size,
                                      C_ptr, ws_ptr, ws_bytes, stream))


def gemm_grouped_sf_raw(A_ptr, act_dtype, offsets, N, K, codes_ptr, scales_ptr, scale_format, bits, group_size,
                        C_ptr, ws_ptr=None, ws_bytes=0, stream=0):
    E = len(offsets) - 1
    arr = (ctypes.c_int32 * (E + 1))(*[int(o) for o in offsets])
    return int(load().fq_gemm_grouped_sf(A_ptr, act_dtype, arr, E, N, K, codes_ptr, scales_ptr, scale_format, bits,
                                         group_size, C_ptr, ws_ptr, ws_bytes, stream))


def zscale_bytes(K, N, group_size):
    return int(load().fq_zscale_bytes(K, N, group_size))


def quantize_w4a8_raw(W_ptr, K, N, group_size, codes_ptr, z_ptr, t_ptr, stream=0):
    return int(load().fq_quantize_w4a8(W_ptr, K, N, group_size, codes_ptr, z_ptr, t_ptr, stream))


def unpack_w4a8_raw(codes_ptr, K, N, q_ptr, stream=0):
    return int(load().fq_unpack_w4a8(codes_ptr, K, N, q_ptr, stream))


def quantize_act_i8_raw(A_ptr, act_dtype, M, K, Aq_ptr, alpha_ptr, stream=0):
    return int(load().fq_quantize_act_i8(A_ptr, act_dtype, M, K, Aq_ptr, alpha_ptr, stream))


def gemm_w4a8_workspace_bytes(M, N, K, group_size):
    return int(load().fq_gemm_w4a8_workspace_bytes(M, N, K, group_size))


def gemm_w4a8_raw(Aq_ptr, alpha_ptr, M, N, K, codes_ptr, z_ptr, t_ptr, group_size, C_ptr, out_dtype, ws_ptr, ws_bytes,
                  stream=0):
    return int(load().fq_gemm_w4a8(Aq_ptr, alpha_ptr, M, N, K, codes_ptr, z_ptr, t_ptr, group_size, C_ptr, out_dtype,
                                   ws_ptr, ws_bytes, stream))


# ------------------------------------------------------------------ torch-tensor conveniences
def _stream():
    import torch

    return torch.cuda.current_stream().cuda_stream


def _check(status, where):
    if status != FQ_OK:
        raise FqError(status, where)


def _act_code(t):
    import torch

    if t.dtype == torch.float16:
        return FQ_F16
    if t.dtype == torch.bfloat16:
        return FQ_BF16
    raise TypeError("activations must be float16 or bfloat16")


def _scale_format_of(scales):
    """The fq_scale_format a scale tensor's dtype stands for."""
    import torch

    if scales.dtype == torch.float16:
        return FQ_SCALE_F16
    if scales.dtype == torch.bfloat16:
        return FQ_SCALE_BF16
    raise TypeError("scales must be float16 or bfloat16")


def quantize(W, bits, group_size, scale_format=FQ_SCALE_F16):
    """W: cuda float16 [K, N] -> (codes uint8 [K*N*bits/8], scales [K/g, N] float16, or bfloat16 for
    scale_format=FQ_SCALE_BF16)."""
    import torch

    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous()
    K, N = W.shape
    g = K if group_size in (0, K) else group_size
    nbytes = codes_bytes(K, N, bits)
    sbytes = scales_bytes(K, N, group_size)
    if nbytes == 0 or sbytes == 0:
        raise FqError(FQ_ERR_INVALID_ARG, "fq_quantize")
    codes = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    sdtype = torch.bfloat16 if scale_format == FQ_SCALE_BF16 else torch.float16
    scales = torch.empty((K // g, N), dtype=sdtype, device=W.device)
    _check(quantize_sf_raw(W.data_ptr(), K, N, bits, group_size, scale_format, codes.data_ptr(), scales.data_ptr(),
                           _stream()), "fq_quantize_sf")
    return codes, scales


def unpack(codes, K, N, bits):
    import torch

    q = torch.empty((K, N), dtype=torch.int8, device=codes.device)
    _check(unpack_raw(codes.data_ptr(), K, N, bits, q.data_ptr(), _stream()), "fq_unpack")
    return q


def choose_group(W, g_start, g_min, alpha):
    import torch

    K, N = W.shape
    ws_bytes = choose_group_workspace_bytes(K, N, g_start, g_min)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=W.device)
    st, g = choose_group_raw(W.data_ptr(), K, N, g_start, g_min, float(alpha), ws.data_ptr(), ws_bytes, _stream())
    _check(st, "fq_choose_group")
    return g


def quant_error(W, codes, scales, bits, group_size):
    """Round-trip error of a quantised matrix: (sum of squared errors, largest absolute error)."""
    import torch

    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous()
    K, N = W.shape
    ws_bytes = quant_error_workspace_bytes(K, N)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=W.device)
    st, sse, mx = quant_error_sf_raw(W.data_ptr(), K, N, bits, group_size, _scale_format_of(scales),
                                     codes.data_ptr(), scales.data_ptr(), ws.data_ptr(), ws_bytes, _stream())
    _check(st, "fq_quant_error_sf")
    return sse, mx


def gemm(A, codes, scales, bits, group_size, out=None, workspace=None):
    """A: cuda [M, K] float16/bfloat16 -> C [M, N] of the same dtype."""
    import torch

    assert A.is_cuda and A.is_contiguous()
    M, K = A.shape
    N = scales.shape[1]
    C = out if out is not None else torch.empty((M, N), dtype=A.dtype, device=A.device)
    need = gemm_workspace_bytes(M, N, K, bits, group_size)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=A.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(gemm_sf_raw(A.data_ptr(), _act_code(A), M, N, K, codes.data_ptr(), scales.data_ptr(),
                       _scale_format_of(scales), bits, group_size, C.data_ptr(), ws_ptr, ws_bytes, _stream()),
           "fq_gemm_sf")
    return C


def gemm_grouped(A, offsets, codes, scales, bits, group_size, N, out=None):
    """A: cuda [rows, K]; codes / scales: the experts' buffers back to back."""
    import torch

    rows, K = A.shape
    C = out if out is not None else torch.empty((rows, N), dtype=A.dtype, device=A.device)
    _check(gemm_grouped_sf_raw(A.data_ptr(), _act_code(A), offsets, N, K, codes.data_ptr(), scales.data_ptr(),
                               _scale_format_of(scales), bits, group_size, C.data_ptr(), None, 0, _stream()),
           "fq_gemm_grouped_sf")
    return C


def quantize_w4a8(W, group_size):
    """W: cuda float16 [K, N] -> (codes uint8 [K*N/2], z uint8 [K/g, N], t float16 [N]) of the integer path."""
    import torch

    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous()
    K, N = W.shape
    g = K if group_size in (0, K) else group_size
    zb = zscale_bytes(K, N, group_size)
    if zb == 0:
        raise FqError(FQ_ERR_UNSUPPORTED, "fq_quantize_w4a8")
    codes = torch.empty(codes_bytes(K, N, 4), dtype=torch.uint8, device=W.device)
    z = torch.empty((K // g, N), dtype=torch.uint8, device=W.device)
    t = torch.empty((N,), dtype=torch.float16, device=W.device)
    _check(quantize_w4a8_raw(W.data_ptr(), K, N, group_size, codes.data_ptr(), z.data_ptr(), t.data_ptr(), _stream()),
           "fq_quantize_w4a8")
    return codes, z, t


def unpack_w4a8(codes, K, N):
    import torch

    q = torch.empty((K, N), dtype=torch.int8, device=codes.device)
    _check(unpack_w4a8_raw(codes.data_ptr(), K, N, q.data_ptr(), _stream()), "fq_unpack_w4a8")
    return q


def quantize_act_i8(A):
    """A: cuda [M, K] float16/bfloat16 -> (Aq int8 [M, K], alpha float32 [M])."""
    import torch

    assert A.is_cuda and A.is_contiguous()
    M, K = A.shape
    Aq = torch.empty((M, K), dtype=torch.int8, device=A.device)
    alpha = torch.empty((M,), dtype=torch.float32, device=A.device)
    _check(quantize_act_i8_raw(A.data_ptr(), _act_code(A), M, K, Aq.data_ptr(), alpha.data_ptr(), _stream()),
           "fq_quantize_act_i8")
    return Aq, alpha


def gemm_w4a8(Aq, alpha, codes, z, t, group_size, out_dtype, out=None, workspace=None):
    """C [M, N] (torch dtype out_dtype: float16 or bfloat16) = alpha * t * (Aq . (q * z))."""
    import torch

    M, K = Aq.shape
    N = t.shape[0]
    C = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=Aq.device)
    need = gemm_w4a8_workspace_bytes(M, N, K, group_size)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=Aq.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(gemm_w4a8_raw(Aq.data_ptr(), alpha.data_ptr(), M, N, K, codes.data_ptr(), z.data_ptr(), t.data_ptr(),
                         group_size, C.data_ptr(), FQ_F16 if out_dtype == torch.float16 else FQ_BF16, ws_ptr, ws_bytes,
                         _stream()), "fq_gemm_w4a8")
    return C
