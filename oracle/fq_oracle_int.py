"""Plain CPU definition of the integer path: int8 activations x int4 weights with integer scales.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

The paper's closing section names, as future work, fine-grained quantisation with int8 activations
and int4 weights whose scales are integers, so that integer instructions can be used (section 5,
"Conclusions and Limitations", last paragraph; the limitation it answers is stated just before:
the published method uses no integer instructions).  The paper gives no formula for it.  The reading
taken here keeps Appendix A's quantiser and section 4.1's groups and changes only what "integer
scales" forces:

R17a  Two-level scale.  The scale of group i of column n is  s[i, n] = z[i, n] * t[n]  with an INTEGER
      z in 1..16 (one byte per group) and one half-precision step t[n] per column (Appendix B's storage
      type).  The codes q are Appendix A's: q = int(w / s) in [-7, 7], ties to even, clamped, the
      quotient in binary32 (z * t is exact in binary32: at most 5 x 11 bits).  Then q * z is an integer of
      at most 7 * 16 = 112 in magnitude: an int8, and the whole sum over k runs in integers.
R17b  t[n] is the smallest binary16 t with 16 * 15 * t >= 2 * max|w| over the column (Appendix A's scale
      equation for the widest group, divided by the largest multiplier, rounded UP to storage precision like
      every stored scale here); z[i, n] is the smallest integer in 1..16 with 15 * z * t >= 2 * max|w| over
      the group.  So s >= Appendix A's scale of the group, and |q * s - w| <= s / 2 holds exactly for every
      weight; groups more than 16 times narrower than the column's widest one are quantised with the
      coarser step t (the price of integer scales).  An all-zero column has t = 0, z = 1, q = 0.
R17c  Activations: Appendix A's quantiser at b = 8 applied to each row (token) with a binary32 scale:
      alpha[m] = the smallest binary32 value with 255 * alpha >= 2 * max|A[m, :]| (the printed scale rounded up
      to its storage type, as for the weights), a[m, k] = clamp(round_half_even(fl32(A[m, k] / alpha[m])),
      -127, 127), the quotient in IEEE binary32.  A zero row has alpha = 0, a = 0.  (The paper does not say how
      the activations would be quantised; one scale per token keeps the product exact per row.)
R17d  Product:  S[m, n] = sum_k a[m, k] * q[k, n] * z[k / g, n]  in exact integers
      (|S| <= K * 127 * 112 < 2^31 for K <= 131072), and  C[m, n] = alpha[m] * t[n] * S[m, n].

Pins (tests/test_oracle_int.py): exact-rational re-derivation of t, z, q, alpha and a on small inputs
including ties, zero groups and columns, subnormals and +-65504; two-sided minimality of t and z; the s/2
bound in exact arithmetic; |q * z| <= 112; Python-integer triple loop for S; special cases that reduce to the
floating-point format (all groups equally wide => z = 16 everywhere and s = 16 t); one-hot activation rows;
the int32 bound; the error of the whole chain against the unquantised product.
"""
from __future__ import annotations

import numpy as np

__all__ = ["ZMAX", "quantize_int_scales", "quantize_activations_int8", "gemm_ref_int", "dequantize_int_scales"]

ZMAX = 16          # largest integer group multiplier: 7 * 16 = 112 fits an int8
QMAX = 7           # 4-bit codes, Appendix A
LEVELS = 15        # 2^4 - 1
AMAX = 127         # 8-bit codes of Appendix A: 2^(8-1) - 1
ALEVELS = 255      # 2^8 - 1


def _smallest_f16_with(L: float, target64: np.ndarray) -> np.ndarray:
    """Smallest non-negative binary16 t with L * t >= target (element-wise; comparisons exact in float64)."""
    t = (target64 / L).astype(np.float16)                      # any nearby starting guess
    up, down = np.float16(np.inf), np.float16(-np.inf)
    while True:
        low = L * t.astype(np.float64) < target64
        if not low.any():
            break
        t = np.where(low, np.nextafter(t, up), t).astype(np.float16)
    while True:
        p = np.nextafter(t, down).astype(np.float16)
        ok = (t > 0) & (p >= 0) & (L * p.astype(np.float64) >= target64)
        if not ok.any():
            break
        t = np.where(ok, p, t).astype(np.float16)
    return t


def quantize_int_scales(W: np.ndarray, group_size: int):
    """Readings R17a / R17b.  W float16 [K, N]  ->  (q int8 [K, N], z uint8 [K/g, N], t float16 [N])."""
    if W.dtype != np.float16 or W.ndim != 2:
        raise ValueError("W must be a 2-D float16 array [K, N]")
    K, N = W.shape
    g = K if group_size in (0, K) else int(group_size)
    if g <= 0 or K % g != 0:
        raise ValueError("group_size must divide K")
    m = np.abs(W).reshape(K // g, g, N).max(axis=1).astype(np.float64)       # [K/g, N] group abs-max (exact)
    t = _smallest_f16_with(float(ZMAX * LEVELS), 2.0 * m.max(axis=0))       # [N]
    t64 = t.astype(np.float64)
    # smallest z in 1..ZMAX with LEVELS * z * t >= 2 m   (LEVELS * z * t is exact in float64)
    z = np.full(m.shape, ZMAX, dtype=np.int64)
    for cand in range(ZMAX - 1, 0, -1):
        ok = LEVELS * cand * t64[None, :] >= 2.0 * m
        z = np.where(ok, cand, z)
    z = np.where(t64[None, :] == 0, 1, z)
    s32 = (z.astype(np.float32) * t.astype(np.float32)[None, :])            # exact: <= 5 x 11 bits
    s_rows = np.repeat(s32, g, axis=0)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = W.astype(np.float32) / s_rows                                   # IEEE binary32 quotient
    r = np.where(s_rows == 0, np.float32(0), r)
    q = np.clip(np.rint(r), -QMAX, QMAX).astype(np.int8)
    return q, z.astype(np.uint8), t


def dequantize_int_scales(q: np.ndarray, z: np.ndarray, t: np.ndarray) -> np.ndarray:
    """q * z * t in float64 (exact)."""
    K = q.shape[0]
    g = K // z.shape[0]
    return q.astype(np.float64) * np.repeat(z.astype(np.float64), g, axis=0) * t.astype(np.float64)[None, :]


def quantize_activations_int8(A: np.ndarray):
    """Reading R17c.  A: the activation values (float16 array, or bfloat16 values held in float32) [M, K]
    -> (a int8 [M, K], alpha float32 [M])."""
    A32 = np.asarray(A, dtype=np.float32)                                   # exact for fp16 / bf16 values
    amax = np.abs(A32).max(axis=1) if A32.shape[1] else np.zeros(A32.shape[0], np.float32)
    target = 2.0 * amax.astype(np.float64)
    alpha = (target / ALEVELS).astype(np.float32)                           # any nearby starting guess
    up, down = np.float32(np.inf), np.float32(-np.inf)
    while True:                                                             # 255 * alpha is exact in float64
        low = ALEVELS * alpha.astype(np.float64) < target
        if not low.any():
            break
        alpha = np.where(low, np.nextafter(alpha, up), alpha).astype(np.float32)
    while True:
        p = np.nextafter(alpha, down).astype(np.float32)
        ok = (alpha > 0) & (p >= 0) & (ALEVELS * p.astype(np.float64) >= target)
        if not ok.any():
            break
        alpha = np.where(ok, p, alpha).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = A32 / alpha[:, None]
    r = np.where(alpha[:, None] == 0, np.float32(0), r)
    a = np.clip(np.rint(r), -AMAX, AMAX).astype(np.int8)
    return a, alpha


def gemm_ref_int(a: np.ndarray, alpha: np.ndarray, q: np.ndarray, z: np.ndarray, t: np.ndarray):
    """Reading R17d.  Returns (S int64 [M, N] exact, C float64 [M, N] = alpha * t * S)."""
    K = q.shape[0]
    if a.shape[1] != K:
        raise ValueError("inner dimensions differ")
    g = K // z.shape[0]
    w8 = q.astype(np.int64) * np.repeat(z.astype(np.int64), g, axis=0)      # |w8| <= 112
    S = a.astype(np.int64) @ w8
    C = alpha.astype(np.float64)[:, None] * t.astype(np.float64)[None, :] * S.astype(np.float64)
    return S, C
