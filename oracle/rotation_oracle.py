"""CPU oracle for the outlier-spreading rotation in front of the activation
quantiser: a Hadamard transform of every group of 128 input features.

TEST INFRASTRUCTURE ONLY.  Plain NumPy; shares no code with the HIP path and is
imported only by tests, the smoke check and the benchmark's CPU-baseline leg.

Where it comes from.  QSpec (arXiv 2410.11305) takes its W4A4 / W4A16 schemes from
existing quantisers and names a rotation-based one among them (Sec. 4.1; related
work, "QuaRot"): activations are multiplied by a Hadamard matrix before they are
quantised, the weights by the same matrix offline, so the product is unchanged
while single large channels are spread over many.  The paper gives no detail; this
is a design of this build, stated here as the definition the HIP path is held to:

  * the rotation is block-diagonal with the quantisation groups: each group of 128
    features is multiplied by H_128 (Sylvester construction, natural order,
    H[i][j] = (-1)^popcount(i & j)) and by 2^-3:   x'_g = x_g H_128 / 8.
    H_128 H_128^T = 128 I, so with weights stored in the rotated basis as
    w'_g = w_g H_128 / 16 the product x' w'^T equals x w^T.  Both factors are powers
    of two: the online one is exact.
  * arithmetic (floating point decides an fp16 value and, after it, an integer code,
    so it is fixed): the fast transform, seven stages h = 1, 2, ..., 64, stage h
    replacing every pair (v[j], v[j+h]) (j with bit h clear) by (v[j] + v[j+h],
    v[j] - v[j+h]) in binary32, then the exact scaling, then one rounding to fp16.
    Every value is a fixed expression tree of binary32 additions, whatever the
    order in which a machine evaluates independent pairs.

Pins (tests/test_oracle_pins.py): equality with the float64 product x H / 8 built
from scipy's Hadamard matrix on inputs whose sums are exact, closeness on general
inputs, the explicit entries (-1)^popcount(i & j) on one-hot rows, the involution
(twice = 2 x), energy (Parseval), and the purpose: the draft-mode output error on
the outlier-channel recipe drops.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

BLOCK = 128


def hadamard128_f16(x: np.ndarray) -> np.ndarray:
    """fp16 [M, K] -> fp16 [M, K]: every group of 128 features times H_128 / 8."""
    x = np.asarray(x)
    if x.dtype != np.float16 or x.ndim != 2 or x.shape[1] % BLOCK:
        raise ValueError("x must be fp16 [M, K] with K a multiple of 128")
    M, K = x.shape
    v = x.astype(np.float32).reshape(M, K // BLOCK, BLOCK)
    h = 1
    while h < BLOCK:
        pairs = v.reshape(M, K // BLOCK, BLOCK // (2 * h), 2, h)
        lo, hi = pairs[..., 0, :], pairs[..., 1, :]
        v = np.stack([(lo + hi).astype(np.float32), (lo - hi).astype(np.float32)], axis=-2)
        h *= 2
    v = v.reshape(M, K) * np.float32(0.125)
    return v.astype(np.float16)
