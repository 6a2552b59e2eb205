"""CPU oracle for the dual-mode W4 linear layer of QSpec (arXiv 2410.11305).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition the HIP
kernels are checked against.  It shares no code with the HIP path and must be
imported only by tests, by the smoke check and by the benchmark's CPU-baseline
leg.  The product never routes through it.

What the paper fixes (Sec. 1, Sec. 3 and Sec. 4.1 "Implementations"):
  * one 4-bit weight tensor is shared by two activation modes; nothing but
    the activation scheme changes between draft and verify (Sec. 3);
  * W4A16: the 4-bit weights are dequantised to fp16 at run time and
    multiplied with fp16 activations (Sec. 1, item (1));
  * W4A4: activations are 4-bit too and the product runs on low-precision
    hardware without going back to high precision first (Sec. 1, item (2));
  * quantisation is group-wise with group size 128 (Sec. 4.1).
The paper gives no formula for the quantiser.  The reading used here
(symmetric two's-complement codes in [-8, 7], weight value = code * fp16
group scale, activation scale = fp32 absmax / 7 by IEEE division, codes by
IEEE division + round-half-to-even + clamp) is this build's documented
choice.

Notation (x: activations, W: weights, y = x W^T):
  x   fp16 [M, K]      qa  int8 codes [M, K]   sa  fp32 [M, G]
  qw  int8 codes [N,K] sw  fp16 [N, G]         G = K / 128
  P   int   [M, N, G]  y   fp16 [M, N]

Pins (tests/test_oracle_pins.py): every function here is checked against
exact rational arithmetic and pure-Python brute force on tiny inputs,
hand-worked examples, and invariants.  No function is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

GROUP = 128


def _check_group(K: int, group: int) -> int:
    if group != GROUP:
        raise ValueError("group size is fixed at 128 (Sec. 4.1)")
    if K <= 0 or K % group:
        raise ValueError("K must be a positive multiple of the group size")
    return K // group


# --------------------------------------------------------------------------
# Canonical nibble packing (two 4-bit codes per byte, low nibble = even k)
# --------------------------------------------------------------------------
def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """int8 codes [R, K] in [-8, 7] -> uint8 [R, K/2]; byte = lo | hi << 4
    where lo is the code at even k and hi the code at k + 1, each kept as its
    4-bit two's-complement pattern."""
    codes = np.asarray(codes)
    if codes.ndim != 2 or codes.shape[1] % 2:
        raise ValueError("codes must be [R, K] with K even")
    u = codes.astype(np.int16) & 0xF
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed: np.ndarray) -> np.ndarray:
    """Inverse of pack_nibbles: uint8 [R, K/2] -> int8 [R, K]."""
    packed = np.asarray(packed, dtype=np.uint8)
    lo = (packed & 0xF).astype(np.int16)
    hi = (packed >> 4).astype(np.int16)
    out = np.empty((packed.shape[0], packed.shape[1] * 2), dtype=np.int16)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    out = np.where(out >= 8, out - 16, out)
    return out.astype(np.int8)


# --------------------------------------------------------------------------
# Activation quantiser (draft mode, Sec. 1 item (2): activations are 4-bit)
# --------------------------------------------------------------------------
def quant_act(x: np.ndarray, group: int = GROUP):
    """Per token, per group of 128 input features:
        a = max |x|                       (fp16 widened to fp32, exact)
        s = a / 7                         (binary32 division, round-to-nearest-even)
        q = clamp(rne(x / s), -8, 7)      (binary32 division, then round half to even)
    An all-zero group has s = 0 and q = 0.
    Returns (codes int8 [M, K], scales fp32 [M, G])."""
    x = np.asarray(x)
    if x.dtype != np.float16 or x.ndim != 2:
        raise ValueError("x must be fp16 [M, K]")
    M, K = x.shape
    G = _check_group(K, group)
    xf = x.astype(np.float32).reshape(M, G, group)
    a = np.max(np.abs(xf), axis=2)                         # fp32, order-free
    s = (a / np.float32(7.0)).astype(np.float32)           # IEEE binary32 divide
    q = np.zeros((M, G, group), dtype=np.float32)
    nz = s > 0
    with np.errstate(divide="ignore", invalid="ignore"):
        t = (xf / s[:, :, None]).astype(np.float32)        # IEEE binary32 divide
    t = np.rint(t)                                         # round half to even
    t = np.clip(t, -8.0, 7.0)
    q[nz] = t[nz]
    return q.reshape(M, K).astype(np.int8), s


# --------------------------------------------------------------------------
# Integer per-group partial sums (what the low-precision matrix units produce)
# --------------------------------------------------------------------------
def partials(qa: np.ndarray, qw: np.ndarray, group: int = GROUP) -> np.ndarray:
    """P[m, n, j] = sum over k in group j of qa[m, k] * qw[n, k], exact.

    The contraction runs as one float64 matmul per group; every product is at
    most 64 and every sum at most 128 * 64 in magnitude, so float64 holds all
    intermediate values exactly and the result is cast back to int32."""
    qa = np.asarray(qa)
    qw = np.asarray(qw)
    M, K = qa.shape
    N, K2 = qw.shape
    if K != K2:
        raise ValueError("qa and qw disagree on K")
    G = _check_group(K, group)
    P = np.empty((M, N, G), dtype=np.int32)
    for j in range(G):
        a = qa[:, j * group:(j + 1) * group].astype(np.float64)
        w = qw[:, j * group:(j + 1) * group].astype(np.float64)
        P[:, :, j] = (a @ w.T).astype(np.int32)
    return P


# --------------------------------------------------------------------------
# W4A4 output (draft mode)
# --------------------------------------------------------------------------
def gemm_w4a4(qa, sa, qw, sw, group: int = GROUP) -> np.ndarray:
    """y[m, n] = fp16( sum_j P[m, n, j] * sa[m, j] * sw[n, j] ), the sum taken
    in float64 and rounded once to fp16 (round-to-nearest-even)."""
    P = partials(qa, qw, group).astype(np.float64)
    sa = np.asarray(sa, dtype=np.float32).astype(np.float64)     # [M, G]
    sw = np.asarray(sw, dtype=np.float16).astype(np.float64)     # [N, G]
    y = np.einsum("mnj,mj,nj->mn", P, sa, sw)
    return y.astype(np.float16)


# --------------------------------------------------------------------------
# W4A16 output (verify mode)
# --------------------------------------------------------------------------
def dequant_weights(qw, sw, group: int = GROUP) -> np.ndarray:
    """w[n, k] = qw[n, k] * sw[n, k // 128] in float64 (no fp16 rounding)."""
    qw = np.asarray(qw)
    N, K = qw.shape
    G = _check_group(K, group)
    sw = np.asarray(sw, dtype=np.float16).astype(np.float64)
    if sw.shape != (N, G):
        raise ValueError("sw must be [N, K/128]")
    return qw.astype(np.float64) * np.repeat(sw, group, axis=1)


def gemm_w4a16(x, qw, sw, group: int = GROUP, round_weights_to_fp16: bool = False) -> np.ndarray:
    """y[m, n] = fp16( sum_k x[m, k] * qw[n, k] * sw[n, k // 128] ), the sum in
    float64, rounded once to fp16.  With round_weights_to_fp16 the dequantised
    weight is first rounded to fp16 (information only: it shows how much of
    the error budget an fp16 weight operand spends); parity is judged against
    the default, unrounded form."""
    x = np.asarray(x)
    if x.dtype != np.float16:
        raise ValueError("x must be fp16")
    w = dequant_weights(qw, sw, group)
    if round_weights_to_fp16:
        w = w.astype(np.float16).astype(np.float64)
    y = x.astype(np.float64) @ w.T
    return y.astype(np.float16)


def gemm_w4a16_columns(x, qw, sw, cols, group: int = GROUP) -> np.ndarray:
    """gemm_w4a16 restricted to the output columns `cols` (for sampled checks
    at sizes where the full product is too slow on a CPU)."""
    cols = np.asarray(cols)
    return gemm_w4a16(x, np.asarray(qw)[cols], np.asarray(sw)[cols], group)


def gemm_w4a4_columns(qa, sa, qw, sw, cols, group: int = GROUP) -> np.ndarray:
    """gemm_w4a4 restricted to the output columns `cols`, in the order given (column n
    of the product uses only row n of the weight codes and scales)."""
    cols = np.asarray(cols)
    return gemm_w4a4(qa, sa, np.asarray(qw)[cols], np.asarray(sw)[cols], group)
