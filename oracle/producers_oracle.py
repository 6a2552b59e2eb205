"""CPU oracle for the two producers of draft-mode activations in a Llama-shaped
decoder block: RMSNorm (input of the q/k/v and of the gate/up projections) and
SiLU(gate) * up (input of the down projection).  In the draft pass of QSpec
(arXiv 2410.11305, Sec. 3.1 "Draft Phase"; Sec. 1: activations are quantised to
4 bit on the fly) each of them is followed immediately by the activation
quantiser; the HIP path fuses the pair into one launch, and this file states what
the fused launch must produce: exactly the quantiser's result on the fp16 tensor
the unfused producer would have written.

TEST INFRASTRUCTURE ONLY.  Plain NumPy; shares no code with the HIP path and is
imported only by tests, the smoke check and the benchmark's CPU-baseline leg.

The paper defines neither operator (they are the model's, Sec. 4.1 uses Llama
checkpoints); the definitions are the textbook ones:
    RMSNorm(x)_k = x_k / sqrt(mean_k(x_k^2) + eps) * w_k
    SiLU(g)      = g / (1 + exp(-g))
Readings (floating point decides an fp16 value and, after it, an integer code, so
both sides fix the arithmetic):
  * statistics and the transcendental in binary64, everything that touches the
    result once in binary32, one final rounding to fp16:
        RMSNorm:  r  = fp32( 1 / sqrt( sum_k(x_k^2) / K + eps ) )        (binary64 inside)
                  h_k = fp16( fp32( (x_k * w_k) * r ) )                  (x_k * w_k is exact in binary32)
        SiLU*up:  s  = fp32( g / (1 + exp(-g)) )                         (binary64 inside)
                  h  = fp16( fp32( s * u ) )
    The binary64 parts are order- or library-dependent in their last bit only; that
    reaches the binary32 value with probability ~1e-8 per element and the fp16 value
    far more rarely.
  * eps is a binary32 argument, widened exactly.
  * the merged gate/up tensor holds the gate in its first I columns and up in its
    last I columns.
  * inf / NaN inputs: unspecified, untested.

Pins (tests/test_oracle_pins.py): closed forms (constant rows, one-hot rows, eps that
makes the denominator a power of two, SiLU at 0, ln 3 and large arguments, the identity
SiLU(g) - SiLU(-g) = g), exact scale invariance at eps = 0, column-order probes, and
PyTorch's own CPU rms_norm / silu in float64 as an independent library routine.  No
function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def rmsnorm_f16(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """fp16 [M, K], fp16 [K], eps -> fp16 [M, K] (arithmetic as stated in the header)."""
    x = np.asarray(x)
    w = np.asarray(w)
    if x.dtype != np.float16 or x.ndim != 2 or w.dtype != np.float16 or w.shape != (x.shape[1],):
        raise ValueError("x must be fp16 [M, K] and w fp16 [K]")
    K = x.shape[1]
    x64 = x.astype(np.float64)
    ms = np.sum(x64 * x64, axis=1) / np.float64(K)                      # squares are exact
    r = (1.0 / np.sqrt(ms + np.float64(np.float32(eps)))).astype(np.float32)
    t = x.astype(np.float32) * w.astype(np.float32)[None, :]            # exact: 11 x 11 significant bits
    u = (t * r[:, None]).astype(np.float32)                             # one binary32 rounding
    return u.astype(np.float16)


def silu_mul_f16(gate_up: np.ndarray) -> np.ndarray:
    """fp16 [M, 2I] (gate | up) -> fp16 [M, I] = SiLU(gate) * up."""
    gate_up = np.asarray(gate_up)
    if gate_up.dtype != np.float16 or gate_up.ndim != 2 or gate_up.shape[1] % 2:
        raise ValueError("gate_up must be fp16 [M, 2I]")
    I = gate_up.shape[1] // 2
    g = gate_up[:, :I].astype(np.float64)
    up = gate_up[:, I:].astype(np.float32)
    with np.errstate(over="ignore"):
        s = (g / (1.0 + np.exp(-g))).astype(np.float32)
    return (s * up).astype(np.float32).astype(np.float16)
