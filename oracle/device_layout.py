"""Byte layouts of the device buffers, written out independently of the HIP code.

TEST INFRASTRUCTURE ONLY (see qspec_oracle.py).  The shared weight tensor of
QSpec (paper Sec. 3: the draft and verify modes read the same 4-bit weights)
is stored on the GPU as a permutation of the canonical nibble-packed codes
plus transposed group scales; the activation codes use the same word format.
These functions restate that layout from its specification so that the blob
the GPU writes can be compared byte for byte.

Layout specification
  word   : eight consecutive codes c0..c7 (k = 8w .. 8w+7) as one little-endian
           32-bit word; 4-bit two's-complement code c_e sits at bit 4*POS[e]
           with POS = (0, 4, 1, 5, 2, 6, 3, 7).
  weights: tiles of 16 rows x 128 k (1024 B); tile (T, g) at byte
           (T*G + g)*1024; inside, the 16 bytes at 16*(16*kb + r), kb = 0..3,
           are four words of row 16T + r: word i covers k%128 in
           [32i + 8kb, 32i + 8kb + 8).
           After all tiles: fp16 scales transposed to [G][N].
  acts   : row-major, 16 words per group; the word of codes k%128 in
           [32i + 8kb, +8) sits at word position 4kb + i of its group.
  acts, widened (the second format of the activation quantiser, for the tiled
           draft-mode kernel): row-major, 128 bytes per group, one int8 = 16 * code
           per code.  The code that the packed format keeps in the low (high)
           nibble of byte b of its group's 64 bytes sits at byte b (64 + b).
"""
from __future__ import annotations

import numpy as np

GROUP = 128
POS = (0, 4, 1, 5, 2, 6, 3, 7)     # bit position / 4 of code e inside its word


def _words(codes: np.ndarray) -> np.ndarray:
    """int8 [R, K] -> uint32 [R, K/8] in the word format above."""
    R, K = codes.shape
    if K % 8:
        raise ValueError("K must be a multiple of 8")
    nib = (codes.astype(np.int64) & 0xF).reshape(R, K // 8, 8)
    w = np.zeros((R, K // 8), dtype=np.int64)
    for e in range(8):
        w |= nib[:, :, e] << (4 * POS[e])
    return w.astype(np.uint32)


def _codes_from_words(words: np.ndarray) -> np.ndarray:
    R, W = words.shape
    w = words.astype(np.int64)
    out = np.empty((R, W, 8), dtype=np.int64)
    for e in range(8):
        out[:, :, e] = (w >> (4 * POS[e])) & 0xF
    out = np.where(out >= 8, out - 16, out)
    return out.reshape(R, W * 8).astype(np.int8)


def pack_words(codes: np.ndarray) -> np.ndarray:
    """Public form of the word packer: int8 [R, K] -> uint32 [R, K/8]."""
    return _words(np.asarray(codes))


def act_bytes(codes: np.ndarray) -> np.ndarray:
    """int8 codes [M, K] -> uint8 [M, K/2] as the activation quantiser stores them."""
    codes = np.asarray(codes)
    M, K = codes.shape
    if K % GROUP:
        raise ValueError("K must be a multiple of 128")
    words = _words(codes).reshape(M, K // GROUP, 4, 4)          # [m, g, i, kb]  (k-word = 4i + kb)
    words = np.ascontiguousarray(words.transpose(0, 1, 3, 2))   # stored at position 4kb + i
    return words.astype("<u4").view(np.uint8).reshape(M, -1)


def act_wide_bytes(codes: np.ndarray) -> np.ndarray:
    """int8 codes [M, K] -> int8 [M, K] in the widened activation format (16 * code)."""
    codes = np.asarray(codes)
    M, K = codes.shape
    if K % GROUP:
        raise ValueError("K must be a multiple of 128")
    G = K // GROUP
    src = codes.astype(np.int16).reshape(M, G, GROUP)
    out = np.zeros((M, G, GROUP), dtype=np.int16)
    for i in range(4):
        for kb in range(4):
            for e in range(8):
                k = 32 * i + 8 * kb + e                       # position inside the group
                word = 4 * kb + i                             # word position in the packed group
                b = 4 * word + POS[e] // 2                    # byte of the packed group holding this code
                half = POS[e] % 2                             # 0: its low nibble, 1: its high nibble
                out[:, :, b + 64 * half] = 16 * src[:, :, k]
    return out.reshape(M, K).astype(np.int8)


def decode_act_wide_bytes(qa8: np.ndarray) -> np.ndarray:
    """Inverse of act_wide_bytes -> int8 codes [M, K]."""
    qa8 = np.asarray(qa8, dtype=np.int8)
    M, K = qa8.shape
    G = K // GROUP
    src = qa8.astype(np.int16).reshape(M, G, GROUP)
    out = np.zeros((M, G, GROUP), dtype=np.int16)
    for i in range(4):
        for kb in range(4):
            for e in range(8):
                b = 4 * (4 * kb + i) + POS[e] // 2
                out[:, :, 32 * i + 8 * kb + e] = src[:, :, b + 64 * (POS[e] % 2)] // 16
    return out.reshape(M, K).astype(np.int8)


def decode_act_bytes(qa: np.ndarray) -> np.ndarray:
    qa = np.ascontiguousarray(qa, dtype=np.uint8)
    M = qa.shape[0]
    words = qa.view("<u4").reshape(M, -1, 4, 4)                 # [m, g, kb, i]
    words = np.ascontiguousarray(words.transpose(0, 1, 3, 2)).reshape(M, -1)
    return _codes_from_words(words)


def weight_blob(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """int8 codes [N, K], fp16 scales [N, G] -> uint8 blob of N*K/2 + 2*N*G bytes."""
    codes = np.asarray(codes)
    scales = np.asarray(scales)
    N, K = codes.shape
    if N % 16 or K % GROUP:
        raise ValueError("N must be a multiple of 16 and K of 128")
    G = K // GROUP
    if scales.shape != (N, G) or scales.dtype != np.float16:
        raise ValueError("scales must be fp16 [N, G]")
    words = _words(codes)                                   # [N, K/8]
    # n = 16T + r ; k-word index inside the row = 16g + 4i + kb
    w5 = words.reshape(N // 16, 16, G, 4, 4)                # [T, r, g, i, kb]
    tiles = np.ascontiguousarray(w5.transpose(0, 2, 4, 1, 3))   # [T, g, kb, r, i]
    code_bytes = tiles.astype("<u4").view(np.uint8).reshape(-1)
    scale_bytes = np.ascontiguousarray(scales.T).view(np.uint8).reshape(-1)
    return np.concatenate([code_bytes, scale_bytes])


def decode_weight_blob(blob: np.ndarray, N: int, K: int):
    """Inverse of weight_blob -> (int8 codes [N, K], fp16 scales [N, G])."""
    G = K // GROUP
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    nb = N * K // 2
    tiles = blob[:nb].view("<u4").reshape(N // 16, G, 4, 16, 4)     # [T, g, kb, r, i]
    words = np.ascontiguousarray(tiles.transpose(0, 3, 1, 4, 2)).reshape(N, K // 8)   # [T, r, g, i, kb]
    scales = blob[nb:nb + 2 * N * G].view(np.float16).reshape(G, N).T
    return _codes_from_words(words), np.ascontiguousarray(scales)


def weight_byte_offset(n: int, k: int, G: int) -> int:
    """Byte of the blob that holds code (n, k) (scalar form of the same spec,
    used by the pin that walks the blob code by code)."""
    T, r = divmod(n, 16)
    g, kk = divmod(k, GROUP)
    i, k32 = divmod(kk, 32)
    kb, e = divmod(k32, 8)
    return (T * G + g) * 1024 + 16 * (16 * kb + r) + 4 * i + POS[e] // 2


def weight_nibble_shift(k: int) -> int:
    """0 if code k is the low nibble of its byte, 4 if the high nibble."""
    return 4 * (POS[k % 8] % 2)
