"""CPU oracle for the two steps that follow the verify pass of QSpec
(arXiv 2410.11305, Sec. 3.1): the greedy acceptance policy and the KV-cache
overwrite.

TEST INFRASTRUCTURE ONLY.  Plain, slow Python/NumPy; shares no code with the
HIP path and is imported only by tests, the smoke check and the benchmark's
CPU-baseline leg.

What the paper fixes (Sec. 3.1):
  * "Verify Phase": the high-precision pass takes the last committed token
    followed by the gamma drafted tokens and returns gamma + 1 next-token
    distributions in one forward pass; drafted tokens are checked in order,
    the first rejection discards every later draft, and the token at the
    rejected position is taken from the high-precision distribution there; if
    every draft is accepted, one more token is taken from distribution
    gamma + 1.
  * "Acceptance Policy": both passes decode greedily; a drafted token is
    accepted exactly when it equals the top-1 token of the high-precision
    distribution at its position.
  * "KV Cache Overwriting": the cache entries the draft pass wrote for accepted
    tokens are replaced by the entries the verify pass computed.

Readings where the paper is silent:
  * top-1 under ties: the lowest token id among the maxima;
  * NaN logits: unspecified, untested;
  * the verify pass's row 0 belongs to the last committed token (its cache entry
    is rewritten too: the verify pass recomputed it at the same precision), rows
    1..a to the accepted drafts; rows after the first rejection are not copied.
    The corrected / bonus token has no cache entry yet: it is the next cycle's
    first input.

Notation: B sequences, gamma drafts each, V vocabulary size;
  logits  [B, gamma+1, V]  verify-pass outputs, row j predicts the token after input j
  draft   [B, gamma]       drafted token ids
  a       [B]              number of accepted drafts, 0..gamma
  out     [B, gamma+1]     the a accepted drafts, then the verify pass's own token; -1 after that

Pins (tests/test_oracle_pins.py): the worked example of the paper's Figure
"mini-sample" (gamma = 4: four accepted plus one extra token, then two accepted
plus one corrected token, so the next cycle starts at the ninth token), an
independent longest-common-prefix formulation, brute force over every small
case, and invariants.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def top1(row: np.ndarray) -> int:
    """Index of the largest logit; the lowest index among equal maxima."""
    best, best_i = None, -1
    for i, v in enumerate(row.tolist()):
        if best is None or v > best:
            best, best_i = v, i
    return best_i


def greedy_accept(logits: np.ndarray, draft: np.ndarray):
    """Sec. 3.1 "Acceptance Policy" with the sequential rule of "Verify Phase".
    Returns (a int32 [B], out int32 [B, gamma+1])."""
    logits = np.asarray(logits)
    draft = np.asarray(draft)
    B, rows, V = logits.shape
    gamma = rows - 1
    if draft.shape != (B, gamma):
        raise ValueError("draft must be [B, gamma] for logits [B, gamma+1, V]")
    a = np.zeros(B, dtype=np.int32)
    out = np.full((B, gamma + 1), -1, dtype=np.int32)
    for b in range(B):
        n = 0
        while n < gamma and top1(logits[b, n]) == int(draft[b, n]):
            out[b, n] = int(draft[b, n])          # accepted
            n += 1
        out[b, n] = top1(logits[b, n])            # corrected token (n < gamma) or the extra one (n == gamma)
        a[b] = n
    return a, out


def kv_overwrite(cache: np.ndarray, kv_verify: np.ndarray, a: np.ndarray, pos: np.ndarray) -> np.ndarray:
    """Sec. 3.1 "KV Cache Overwriting": a copy of `cache` [B, S, D] in which, for every
    sequence b, rows pos[b] .. pos[b] + a[b] are replaced by rows 0 .. a[b] of
    kv_verify [B, gamma+1, D].  Rows that would fall outside the cache are skipped."""
    cache = np.array(cache, copy=True)
    B, S, D = cache.shape
    for b in range(B):
        for j in range(int(a[b]) + 1):
            s = int(pos[b]) + j
            if 0 <= s < S:
                cache[b, s, :] = kv_verify[b, j, :]
    return cache
