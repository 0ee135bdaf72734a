"""Plain CPU definition of FineQuant's weight-only quantised linear layer.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

What is defined here, and the passage of the paper each part follows:

* ``quantize``      linear abs-max symmetric quantiser, Appendix A (the two
                    equations under "Linear quantization with absolute
                    maximum"), applied to contiguous blocks of ``g`` elements
                    inside a column (section 4.1, "Quantization Method"), with
                    the scaling factors stored in half precision (Appendix B).
* ``dequantize``    A' = Q x s, Appendix A.
* ``gemm_ref``      the plain definition of the product the fused kernels
                    compute (section 4.1, "GPU kernel implementations"):
                    C = A . dequant(W), evaluated in fp64.
* ``choose_group``  the adaptive fine-grained heuristic of section 3.3.
* ``quant_error``   the quantisation error the paper plots against the group
                    size (section 3.2, figure 2a: mean squared error between
                    the weights and their quantise-dequantise round trip):
                    sum and maximum of (w - q*s)^2 / |w - q*s| in fp64.

Readings taken where the paper is silent or ambiguous (each one is listed in
the design notes of the repository as well):

R1  Step constant: s = 2*max|w| / (2^b - 1), exactly as printed, i.e. the
    interval [-max, max] is tiled by 2^b - 1 equal bins; codes lie in
    [-(2^(b-1)-1), 2^(b-1)-1].
R2  ``int(.)`` is round-to-nearest, ties to even, followed by a clamp to the
    code range (only the group's extreme element can reach the clamp).
R3  The stored scale is the smallest half-precision number s with
    (2^b - 1) * s >= 2 * max|w| (the printed value rounded *up* to storage
    precision), and codes are computed with that stored scale.  This makes
    |q*s - w| <= s/2 hold exactly for every element.
R4  The quotient w / s is evaluated in IEEE binary32 (correctly rounded
    division).  For half-precision operands this gives the same code as exact
    rational arithmetic; a test proves that on an exhaustive window.
R5  An all-zero group has s = 0 and q = 0.
R6  Section 3.3: "range" is the abs-max of a group; a halving step is taken
    while, for ANY parent group, the smaller of its two children's ranges
    differs from the parent's by more than alpha in relative terms:
    min(child ranges) < (1 - alpha) * parent range.  (Read literally with
    abs-max ranges, new/old > alpha is always true for alpha < 1 because the
    child that holds the parent's maximum has ratio exactly 1; the closing
    sentence of the section states the stop rule in terms of the range
    difference between two granularities falling below alpha, which is what
    is implemented.)  One group size per
    matrix.  The value of alpha is not recoverable from the paper (its figure
    2b is an image): the *default* alpha is PARITY UNPINNED; the function
    alpha -> g is pinned by constructed cases.

R8  Code widths.  Appendix A is written for any bit width b; section 4.2 and
    Table 5 evaluate 8, 4 and 3 bits (3 bits for accuracy only, the paper has
    no 3-bit kernel).  b = 3 gives codes in [-3, 3] and the denominator 7; the
    footprints Table 5 prints for its int3 rows follow from 3 + 16/g bits per
    weight, i.e. from a true 3-bit packing.

R7  Scale format.  Appendix B stores the scales in half precision; section
    4.1 ("GPU kernel implementations") describes kernels whose scales have the
    data type of the activation, i.e. bfloat16 scales next to bfloat16
    activations.  ``scale_format="bf16"`` is that variant: the stored scale
    is the smallest *bfloat16* number s with (2^b - 1) * s >= 2 * max|w|;
    everything else (binary32 quotient, ties to even, clamp) is unchanged, so
    |q*s - w| <= s/2 still holds exactly.  Such scales are returned as
    float32 arrays whose low 16 bits are zero (numpy has no bfloat16).

Pins (tests marked "not gpu"): exact-rational brute force for scales and
codes, the s/2 reconstruction bound, code range, g = K against an
independently written per-column quantiser, sign symmetry, power-of-two
equivariance, child-scale <= parent-scale, the footprint closed form against
the paper's Table 5, brute-force dot products, one-hot and all-ones GEMM
special cases, and constructed matrices with a known heuristic answer; for ``quant_error``:
a hand-computed column, the zero error of exactly representable weights, the
s/2 bound and the (sum of s^2)/12-per-weight expectation on uniformly spread
weights; for the bfloat16 scale format: exact-rational minimality of every
scale over all binary16 abs-max values, the bit pattern (low 16 bits zero),
exact-rational codes on an exhaustive window, the s/2 bound, power-of-two
equivariance and the bracket f16-format scale <= bf16-format scale < f16-format
scale * (1 + 2^-7) that the two roundings of one real number must obey.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "qmax_of",
    "levels_of",
    "group_absmax",
    "scale_from_absmax",
    "quantize",
    "dequantize",
    "gemm_ref",
    "gemm_ref_grouped",
    "choose_group",
    "bits_per_weight",
    "quant_error",
    "bf16_scale_bits",
]


def qmax_of(bits: int) -> int:
    """Largest code magnitude, 2^(b-1) - 1 (3 for int3, 7 for int4, 127 for int8)."""
    if bits not in (3, 4, 8):
        raise ValueError("bits must be 3, 4 or 8")
    return (1 << (bits - 1)) - 1


def levels_of(bits: int) -> int:
    """The denominator 2^b - 1 of Appendix A's scale equation."""
    if bits not in (3, 4, 8):
        raise ValueError("bits must be 3, 4 or 8")
    return (1 << bits) - 1


def _check_w(W: np.ndarray, group_size: int) -> int:
    if W.dtype != np.float16 or W.ndim != 2:
        raise ValueError("W must be a 2-D float16 array [K, N]")
    K = W.shape[0]
    g = K if group_size in (0, K) else int(group_size)
    if g <= 0 or K % g != 0:
        raise ValueError("group_size must divide K")
    return g


def group_absmax(W: np.ndarray, group_size: int) -> np.ndarray:
    """max |w| over each block of ``g`` consecutive rows of each column.

    Section 4.1: each contiguous block of B elements in a given column has its
    own scaling factor.  Returns float16 [K/g, N] (exact: a maximum of halves).
    """
    g = _check_w(W, group_size)
    K, N = W.shape
    return np.abs(W).reshape(K // g, g, N).max(axis=1)


def _bf16_step(s: np.ndarray, up: bool) -> np.ndarray:
    """Neighbouring bfloat16 value of a non-negative bfloat16 held in float32."""
    b = s.view(np.uint32).astype(np.int64)
    b = b + 0x10000 if up else b - 0x10000
    return b.astype(np.uint32).view(np.float32)


def scale_from_absmax(m: np.ndarray, bits: int, scale_format: str = "f16") -> np.ndarray:
    """Smallest storable ``s >= 0`` with (2^b - 1) * s >= 2 * m  (readings R3, R7).

    Appendix A gives s = 2*max / (2^b - 1); Appendix B says it is stored in
    half precision (``scale_format="f16"``, returned as float16); section 4.1's
    kernels for bfloat16 activations take bfloat16 scales
    (``scale_format="bf16"``, returned as float32 with the low 16 bits zero).
    The comparison is done in float64, where both sides are exact (an 8-bit
    integer times a significand of at most 11 bits; a doubling).
    """
    if m.dtype != np.float16:
        raise ValueError("abs-max must be float16")
    if scale_format not in ("f16", "bf16"):
        raise ValueError("scale_format must be 'f16' or 'bf16'")
    L = float(levels_of(bits))
    target = 2.0 * m.astype(np.float64)
    if scale_format == "bf16":
        # any nearby bfloat16 starting guess will do: drop the low half of the binary32 quotient
        guess = (target / L).astype(np.float32)
        s = (guess.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
        while True:
            low = L * s.astype(np.float64) < target
            if not low.any():
                break
            s = np.where(low, _bf16_step(s, True), s).astype(np.float32)
        while True:
            pos = s > 0
            p = np.where(pos, _bf16_step(np.where(pos, s, np.float32(1.0)), False), s).astype(np.float32)
            ok = pos & (L * p.astype(np.float64) >= target)
            if not ok.any():
                break
            s = np.where(ok, p, s).astype(np.float32)
        return s
    s = (target / L).astype(np.float16)  # any nearby starting guess will do
    pos_inf = np.float16(np.inf)
    neg_inf = np.float16(-np.inf)
    # walk up while too small
    while True:
        low = L * s.astype(np.float64) < target
        if not low.any():
            break
        s = np.where(low, np.nextafter(s, pos_inf), s).astype(np.float16)
    # walk down while the predecessor (kept non-negative) still satisfies it
    while True:
        p = np.nextafter(s, neg_inf).astype(np.float16)
        ok = (s > 0) & (p >= 0) & (L * p.astype(np.float64) >= target)
        if not ok.any():
            break
        s = np.where(ok, p, s).astype(np.float16)
    return s


def bf16_scale_bits(s: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of bfloat16 scales held in float32 (low halves must be zero)."""
    b = np.ascontiguousarray(s, dtype=np.float32).view(np.uint32)
    if np.any(b & np.uint32(0xFFFF)):
        raise ValueError("not bfloat16 values")
    return (b >> np.uint32(16)).astype(np.uint16)


def quantize(W: np.ndarray, bits: int, group_size: int, scale_format: str = "f16"):
    """Appendix A's encoder on blocks of ``g`` rows per column.

    Returns ``(q, s)``: int8 codes [K, N] and scales [K/g, N] (float16, or for
    ``scale_format="bf16"`` bfloat16 values held in float32).
    ``group_size`` 0 or K means one scale per column.
    """
    g = _check_w(W, group_size)
    K, N = W.shape
    qm = qmax_of(bits)
    s = scale_from_absmax(group_absmax(W, g), bits, scale_format)   # [K/g, N]
    s_rows = np.repeat(s.astype(np.float32), g, axis=0)        # [K, N]   f32
    w32 = W.astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = w32 / s_rows                                        # IEEE binary32
    r = np.where(s_rows == 0, np.float32(0), r)
    q = np.clip(np.rint(r), -qm, qm).astype(np.int8)           # ties to even
    return q, s


def dequantize(q: np.ndarray, s: np.ndarray) -> np.ndarray:
    """A' = Q x s (Appendix A), exact in float64.  q [K,N], s [K/g,N]."""
    K, N = q.shape
    G = s.shape[0]
    if K % G != 0 or s.shape[1] != N:
        raise ValueError("scale matrix does not match the codes")
    g = K // G
    return q.astype(np.float64) * np.repeat(s.astype(np.float64), g, axis=0)


def gemm_ref(A: np.ndarray, q: np.ndarray, s: np.ndarray, col_block: int = 2048) -> np.ndarray:
    """C = A . dequant(q, s) in float64, by blocks of columns to bound memory.

    A holds the activation values exactly as given (fp16 values, or bf16
    values carried in a wider float array).
    """
    A64 = np.asarray(A, dtype=np.float64)
    M, K = A64.shape
    if q.shape[0] != K:
        raise ValueError("inner dimensions differ")
    N = q.shape[1]
    C = np.empty((M, N), dtype=np.float64)
    for n0 in range(0, N, col_block):
        n1 = min(N, n0 + col_block)
        C[:, n0:n1] = A64 @ dequantize(q[:, n0:n1], s[:, n0:n1])
    return C


def gemm_ref_grouped(A: np.ndarray, offsets, qs, ss) -> np.ndarray:
    """Expert-by-expert product for a mixture-of-experts layer.

    Rows offsets[e]:offsets[e+1] of A (tokens already sorted by expert) are
    multiplied by expert e's dequantised matrix; experts with no rows are
    skipped.  ``qs`` / ``ss`` are sequences of per-expert codes and scales.
    """
    A64 = np.asarray(A, dtype=np.float64)
    N = qs[0].shape[1]
    C = np.zeros((A64.shape[0], N), dtype=np.float64)
    for e in range(len(qs)):
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        if r1 > r0:
            C[r0:r1] = gemm_ref(A64[r0:r1], qs[e], ss[e])
    return C


def choose_group(W: np.ndarray, g_start: int, g_min: int, alpha: float) -> int:
    """Adaptive fine-grained group size for one matrix (section 3.3, reading R6).

    Start at ``g_start`` (0 = one group per column).  While the halved size is
    allowed (an integer, >= g_min), compute for every parent group the ranges
    (abs-max) of its two halves; if for any parent
    ``min(child ranges) < (1 - alpha) * parent range`` the size is halved and
    the test repeated, otherwise the current size is returned.  The comparison
    is carried out in binary32: thr = fl(1 - alpha), then
    ``min_child < fl(thr * parent)``.
    """
    if W.dtype != np.float16 or W.ndim != 2:
        raise ValueError("W must be a 2-D float16 array [K, N]")
    K, N = W.shape
    g = K if g_start in (0, K) else int(g_start)
    if g <= 0 or K % g != 0 or g_min <= 0:
        raise ValueError("bad group sizes")
    thr = np.float32(1.0) - np.float32(alpha)
    absW = np.abs(W)
    while g % 2 == 0 and g // 2 >= g_min:
        h = g // 2
        child = absW.reshape(K // h, h, N).max(axis=1).astype(np.float32)   # [K/h, N]
        c0 = child[0::2]
        c1 = child[1::2]
        parent = np.maximum(c0, c1)
        small = np.minimum(c0, c1)
        if np.any(small < (thr * parent).astype(np.float32)):
            g = h
        else:
            break
    return g


def bits_per_weight(bits: int, group_size: int) -> float:
    """Storage per weight: b bits of code plus one 16-bit scale per group.

    Follows from section 4.1 (one scaling factor per block of B elements) and
    Appendix B (half-precision scales); Table 5's footprints obey it.
    """
    return bits + 16.0 / group_size


def quant_error(W: np.ndarray, q: np.ndarray, s: np.ndarray):
    """Sum of squared errors and largest absolute error of the round trip.

    Section 3.2 measures quantisation quality as the mean squared error
    between a weight matrix and its dequantised codes (the MSE axis of figure
    2a); Appendix A defines the dequantised value as Q x s.  Everything is
    exact in fp64 up to the final additions: w is binary16, q an integer of at
    most 8 bits and s binary16, so q*s and w - q*s are exact.

    Returns ``(sse, max_abs)``; the mean squared error is ``sse / W.size``.
    """
    W = np.asarray(W)
    err = W.astype(np.float64) - dequantize(q, s)
    return float(np.sum(err * err)), float(np.max(np.abs(err))) if err.size else 0.0
