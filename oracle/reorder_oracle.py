"""CPU oracle for the reordering activation quantiser: outlier channels are moved
to the last groups of the input dimension and those groups are quantised with
about 8 bits, carried as two 4-bit groups each.

TEST INFRASTRUCTURE ONLY.  Plain NumPy; shares no code with the HIP path and is
imported only by tests, the smoke check and the benchmark's CPU-baseline leg.

Where it comes from.  QSpec (arXiv 2410.11305) builds on existing 4-bit quantisers
(Sec. 4.1) and names one that reorders channels so that the few large ones sit
together and keeps those in higher precision (related work, "Atom").  The paper gives
no detail; this is a design of this build, stated here as the definition the HIP
path is held to.  It needs no change to the draft-mode GEMM:

  * perm[p] is the input channel that sits at position p of the reordered tensor
    (chosen offline from calibration data; the weights' columns are reordered the
    same way before they are quantised and packed).  The last G_o groups of the
    reordered tensor are the outlier groups.
  * groups 0 .. G - G_o - 1 are quantised like any activation group:
    a = max|x|, s = a / 7, q = clamp(rne(x / s), -8, 7)         (binary32, IEEE division)
  * an outlier group is quantised to 239 levels,
    a = max|x|, s = a / 119, q8 = clamp(rne(x / s), -119, 119)  (binary32, IEEE division)
    and written as TWO 4-bit groups that multiply the same weight group:
        q8 = 16 * hi + lo,   lo = ((q8 + 8) mod 16) - 8 in [-8, 7],   hi in [-7, 7]
        group "hi": codes hi, scale 16 * s (exact);   group "lo": codes lo, scale s
    119 = 16 * 7 + 7 is the largest magnitude whose high digit fits a 4-bit code.
    The output therefore has G' = G + G_o groups (K' = K + 128 G_o): the ordinary
    groups in order, then hi, lo of each outlier group; the weight tensor holds each
    outlier group twice in the same places.  sum_k q8 s w = sum_k hi (16 s) w + sum_k lo s w.
  * an all-zero group has s = 0 and codes 0, as everywhere.

Pins (tests/test_oracle_pins.py): a hand-worked group (tests/golden/), brute force in
exact rational arithmetic, the digit identity 16 hi + lo = q8 over the whole range,
equality of the ordinary groups with the plain quantiser on the gathered tensor, the
product identity with duplicated weight groups in exact integers, and the purpose (the
draft-mode output error on the outlier recipe).  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

GROUP = 128
LEVELS = 119          # 16 * 7 + 7


def reorder_quant(x: np.ndarray, perm: np.ndarray, n_outlier_groups: int):
    """x fp16 [M, K], perm int [K] (a permutation), G_o -> (codes int8 [M, K + 128 G_o],
    scales fp32 [M, G + G_o])."""
    x = np.asarray(x)
    perm = np.asarray(perm)
    if x.dtype != np.float16 or x.ndim != 2 or x.shape[1] % GROUP:
        raise ValueError("x must be fp16 [M, K] with K a multiple of 128")
    M, K = x.shape
    G = K // GROUP
    Go = int(n_outlier_groups)
    if not 0 <= Go <= G or sorted(perm.tolist()) != list(range(K)):
        raise ValueError("perm must be a permutation of range(K) and 0 <= n_outlier_groups <= K / 128")
    xr = x[:, perm].astype(np.float32).reshape(M, G, GROUP)
    codes = np.zeros((M, G + Go, GROUP), dtype=np.int8)
    scales = np.zeros((M, G + Go), dtype=np.float32)
    a = np.max(np.abs(xr), axis=2)
    for g in range(G):
        outlier = g >= G - Go
        div = np.float32(LEVELS if outlier else 7)
        lim_lo, lim_hi = (-LEVELS, LEVELS) if outlier else (-8, 7)
        s = (a[:, g] / div).astype(np.float32)
        with np.errstate(divide="ignore", invalid="ignore"):
            t = np.rint((xr[:, g, :] / s[:, None]).astype(np.float32))
        q = np.where(s[:, None] > 0, np.clip(t, lim_lo, lim_hi), 0.0).astype(np.int32)
        if not outlier:
            codes[:, g, :] = q
            scales[:, g] = s
        else:
            t_ = g - (G - Go)
            lo = ((q + 8) % 16) - 8
            hi = (q - lo) // 16
            codes[:, G - Go + 2 * t_, :] = hi
            codes[:, G - Go + 2 * t_ + 1, :] = lo
            scales[:, G - Go + 2 * t_] = s * np.float32(16.0)
            scales[:, G - Go + 2 * t_ + 1] = s
    return codes.reshape(M, (G + Go) * GROUP), scales


def expand_weight_columns(w: np.ndarray, perm: np.ndarray, n_outlier_groups: int) -> np.ndarray:
    """Columns of a [N, K] array in the order the quantised activations use: reordered by
    perm, each of the last G_o groups twice in a row.  (Offline step on the weights;
    works on codes as well as on real values.)"""
    w = np.asarray(w)
    N, K = w.shape
    G, Go = K // GROUP, int(n_outlier_groups)
    wr = w[:, np.asarray(perm)].reshape(N, G, GROUP)
    parts = [wr[:, :G - Go, :].reshape(N, -1)]
    for g in range(G - Go, G):
        parts += [wr[:, g, :], wr[:, g, :]]
    return np.concatenate(parts, axis=1)
