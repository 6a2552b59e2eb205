"""Pins for the CPU oracle: every function in oracle/ is checked against
something other than itself -- exact rational arithmetic, pure-Python brute
force, hand-worked examples (tests/golden/) and invariants of the definitions.
No GPU needed."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import device_layout as lay
from oracle import qspec_oracle as orc
from paper_2410_11305_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- exact helpers
def _round_half_even(fr: Fraction) -> int:
    return round(fr)          # Fraction.__round__ rounds half to even


def _fl(fr: Fraction, mant_bits: int, emin: int) -> Fraction:
    """Nearest binary float (round-to-nearest-even) with `mant_bits` stored
    mantissa bits and minimum normal exponent `emin`, as an exact Fraction
    (overflow is not handled: never reached in these tests)."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, emin)
    ulp = Fraction(2) ** (e - mant_bits)
    return sign * _round_half_even(a / ulp) * ulp


def fl32(fr):
    return _fl(fr, 23, -126)


def fl16(fr):
    return _fl(fr, 10, -14)


def F(v) -> Fraction:
    return Fraction(float(v))


def exact_quant_group(xs):
    """One group by the stated rule in exact arithmetic with explicit binary32
    roundings of the two divisions."""
    fx = [F(v) for v in xs]
    a = max(abs(v) for v in fx)
    if a == 0:
        return Fraction(0), [0] * len(xs)
    s = fl32(a / 7)
    q = []
    for v in fx:
        t = fl32(v / s)
        q.append(int(min(7, max(-8, _round_half_even(t)))))
    return s, q


# ---------------------------------------------------------------- inputs
def _tiny_x(seed, M, K):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 3, replace=False)] *= 20
    return x.astype(np.float16)


# ================================================================ O1 packing
def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line)
    return rows


def test_canonical_pack_hand_examples():
    for row in _read_golden("nibble_words.txt"):
        kind, rest = row.split(":", 1)
        lhs, rhs = rest.split("->")
        codes = np.array([[int(v) for v in lhs.split()]], dtype=np.int8)
        want = int(rhs.strip(), 16)
        if kind == "canonical":
            assert int(orc.pack_nibbles(codes)[0, 0]) == want
        else:
            assert int(lay.pack_words(codes)[0, 0]) == want


def test_canonical_pack_roundtrip_all_pairs():
    vals = np.arange(-8, 8, dtype=np.int8)
    codes = np.array([[a, b] for a in vals for b in vals], dtype=np.int8)
    packed = orc.pack_nibbles(codes)
    assert packed.shape == (256, 1)
    assert len(set(packed[:, 0].tolist())) == 256          # a bijection on bytes
    assert np.array_equal(orc.unpack_nibbles(packed), codes)


def test_weight_blob_matches_scalar_walk():
    """Vectorised blob builder against a code-by-code walk of the layout rule."""
    N, K = 48, 384
    G = K // 128
    rng = np.random.default_rng(5)
    codes = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    scales = rng.uniform(0.002, 0.01, size=(N, G)).astype(np.float16)
    blob = lay.weight_blob(codes, scales)
    assert blob.size == N * K // 2 + 2 * N * G
    seen = np.zeros(N * K // 2, dtype=np.int32)
    for n in range(N):
        for k in range(K):
            off = lay.weight_byte_offset(n, k, G)
            sh = lay.weight_nibble_shift(k)
            nib = (int(blob[off]) >> sh) & 0xF
            assert nib == (int(codes[n, k]) & 0xF), (n, k)
            seen[off] += 1
    assert np.all(seen == 2)                                # every byte holds two codes
    sc = blob[N * K // 2:].view(np.float16).reshape(G, N)
    for n in range(N):
        for g in range(G):
            assert sc[g, n] == scales[n, g]


def test_weight_blob_roundtrip_and_tile_locality():
    N, K = 64, 512
    G = K // 128
    codes, scales, _ = synth.generic_case(11, 1, N, K)
    blob = lay.weight_blob(codes, scales)
    c2, s2 = lay.decode_weight_blob(blob, N, K)
    assert np.array_equal(c2, codes)
    assert np.array_equal(s2.view(np.uint16), scales.view(np.uint16))
    # the 1024 bytes of tile (T, g) hold exactly rows 16T..16T+15, group g
    for T in range(N // 16):
        for g in range(G):
            tile = blob[(T * G + g) * 1024:(T * G + g + 1) * 1024]
            nibs = np.concatenate([tile & 0xF, tile >> 4])
            want = (codes[16 * T:16 * T + 16, 128 * g:128 * g + 128].astype(np.int16) & 0xF).ravel()
            assert np.array_equal(np.sort(nibs), np.sort(want))


def test_act_bytes_roundtrip_and_word_order():
    rng = np.random.default_rng(2)
    codes = rng.integers(-8, 8, size=(5, 256), dtype=np.int8)
    b = lay.act_bytes(codes)
    assert b.shape == (5, 128) and b.dtype == np.uint8
    assert np.array_equal(lay.decode_act_bytes(b), codes)
    # word of codes [32i + 8kb, +8) of group g sits at word position 16g + 4kb + i
    words = lay.pack_words(codes)
    stored = b.view("<u4")
    for m in range(5):
        for g in range(2):
            for i in range(4):
                for kb in range(4):
                    assert stored[m, 16 * g + 4 * kb + i] == words[m, 16 * g + 4 * i + kb]


def test_act_wide_bytes_against_the_packed_bytes_nibble_by_nibble():
    """The widened activation format is defined through the packed one: the code in the
    low (high) nibble of byte b of a packed group is 16 * code at byte b (64 + b) of the
    widened group.  Checked by a scalar walk over the packed bytes, a round trip, a
    hand-written group and two planted mistakes (halves swapped; low and high taken
    from the wrong nibble)."""
    rng = np.random.default_rng(12)
    codes = rng.integers(-8, 8, size=(3, 384), dtype=np.int8)
    wide = lay.act_wide_bytes(codes)
    assert wide.shape == (3, 384) and wide.dtype == np.int8
    packed = lay.act_bytes(codes)

    def signed(n):
        return n - 16 if n >= 8 else n

    def walk(packed, lo_first=True, swap_nibbles=False):
        out = np.zeros((packed.shape[0], packed.shape[1] * 2), dtype=np.int8)
        for m in range(packed.shape[0]):
            for g in range(packed.shape[1] // 64):
                for b in range(64):
                    byte = int(packed[m, 64 * g + b])
                    lo, hi = signed(byte & 15), signed(byte >> 4)
                    if swap_nibbles:
                        lo, hi = hi, lo
                    out[m, 128 * g + (b if lo_first else 64 + b)] = 16 * lo
                    out[m, 128 * g + (64 + b if lo_first else b)] = 16 * hi
        return out

    assert np.array_equal(wide, walk(packed))
    assert not np.array_equal(wide, walk(packed, lo_first=False))
    assert not np.array_equal(wide, walk(packed, swap_nibbles=True))
    assert np.array_equal(lay.decode_act_wide_bytes(wide), codes)
    # every group holds exactly its 128 codes, times 16
    for m in range(3):
        for g in range(3):
            assert np.array_equal(np.sort(wide[m, 128 * g:128 * g + 128].astype(np.int16)),
                                  np.sort(16 * codes[m, 128 * g:128 * g + 128].astype(np.int16)))
    # by hand: codes k = 0..7 of a group are word (i = 0, kb = 0) -> packed word position 0, i.e.
    # packed bytes 0..3 = (c2 c0), (c6 c4), (c3 c1), (c7 c5) as (high low) nibbles
    one = np.zeros((1, 128), dtype=np.int8)
    one[0, :8] = [1, 2, 3, 4, 5, 6, 7, -8]
    w = lay.act_wide_bytes(one)[0].astype(np.int16)
    assert w[0:4].tolist() == [16 * 1, 16 * 5, 16 * 2, 16 * 6]            # low nibbles: c0 c4 c1 c5
    assert w[64:68].tolist() == [16 * 3, 16 * 7, 16 * 4, 16 * -8]         # high nibbles: c2 c6 c3 c7
    assert int(np.count_nonzero(w)) == 8
    # codes k = 8..15 (i = 0, kb = 1) go to word position 4: bytes 16..19 and 80..83
    two = np.zeros((1, 128), dtype=np.int8)
    two[0, 8:16] = [1, 2, 3, 4, 5, 6, 7, -8]
    w = lay.act_wide_bytes(two)[0].astype(np.int16)
    assert w[16:20].tolist() == [16, 80, 32, 96] and w[80:84].tolist() == [48, 112, 64, -128]


# ================================================================ O2 quant_act
def test_quant_act_hand_example_half_even():
    rows = dict(r.split(":", 1) for r in _read_golden("quant_act_rounding.txt"))
    vals = [float(v) for v in rows["values"].split()]
    want = [int(v) for v in rows["codes"].split()]
    x = np.zeros((1, 128), dtype=np.float16)
    x[0, :len(vals)] = vals
    q, s = orc.quant_act(x)
    assert s.dtype == np.float32 and s.shape == (1, 1)
    assert float(s[0, 0]) == float(rows["scale"])
    assert q[0, :len(vals)].tolist() == want
    assert not q[0, len(vals):].any()


def test_quant_act_matches_exact_rational_arithmetic():
    M, K = 3, 256
    x = _tiny_x(7, M, K)
    # plant exact ties and extremes in one group: scale is exactly 0.25
    x[1, 128:] = 0
    x[1, 128:136] = np.array([1.75, -0.875, 0.125, 0.375, 0.625, -0.125, -0.625, 0.875], np.float16)
    q, s = orc.quant_act(x)
    for m in range(M):
        for j in range(K // 128):
            s_ex, q_ex = exact_quant_group(x[m, 128 * j:128 * j + 128])
            assert F(s[m, j]) == s_ex, (m, j)
            assert q[m, 128 * j:128 * j + 128].tolist() == q_ex, (m, j)
    assert q[1, 128:136].tolist() == [7, -4, 0, 2, 2, 0, -2, 4]


def test_quant_act_exact_on_benchmark_activations_separates_reciprocal():
    """All 8 x 4096 draft activations of configuration 2 in exact arithmetic.
    The set contains values where x * (1/s) rounds to a different code than
    the true quotient x / s, so a reciprocal-multiply shortcut fails here."""
    x = synth.activations(2, 0, 8, 4096, verify=False)
    q, s = orc.quant_act(x)
    for m in range(8):
        for j in range(32):
            s_ex, q_ex = exact_quant_group(x[m, 128 * j:128 * j + 128])
            assert F(s[m, j]) == s_ex, (m, j)
            assert q[m, 128 * j:128 * j + 128].tolist() == q_ex, (m, j)
    xf = x.astype(np.float32).reshape(8, 32, 128)
    shortcut = np.rint(xf * (np.float32(1) / s)[:, :, None]).reshape(8, 4096)
    assert np.count_nonzero(shortcut != q) >= 1


def test_quant_act_fp16_extremes_exact():
    """Largest and smallest fp16 magnitudes, where a wrong precision or a
    reciprocal-multiply would first show."""
    x = np.zeros((2, 128), dtype=np.float16)
    x[0, :4] = [65504, -65504, 32752, 4678]
    x[1, :4] = np.array([6e-8, 1.2e-7, -6e-8, 2.4e-7], dtype=np.float16)   # subnormal fp16
    q, s = orc.quant_act(x)
    for m in range(2):
        s_ex, q_ex = exact_quant_group(x[m])
        assert F(s[m, 0]) == s_ex
        assert q[m].tolist() == q_ex


def test_quant_act_invariants():
    cfg = 2
    K = 4096
    x = synth.activations(cfg, 0, 8, K, verify=False)
    q, s = orc.quant_act(x)
    G = K // 128
    assert q.dtype == np.int8 and q.shape == (8, K) and s.shape == (8, G)
    # reachable range is [-7, 7]: |x/s| <= 7(1 + 2^-23)
    assert q.min() >= -7 and q.max() <= 7
    xf = x.astype(np.float64).reshape(8, G, 128)
    qg = q.reshape(8, G, 128)
    # the absmax element maps to +-7, signs agree, error at most half a step
    idx = np.argmax(np.abs(xf), axis=2)
    top = np.take_along_axis(qg, idx[:, :, None], axis=2)[:, :, 0]
    assert np.all(np.abs(top) == 7)
    assert np.all((np.sign(qg) == np.sign(xf)) | (qg == 0))
    err = np.abs(xf - qg * s.astype(np.float64)[:, :, None])
    assert np.all(err <= 0.5 * s.astype(np.float64)[:, :, None] * (1 + 2.0 ** -22))
    # scaling by a power of two scales s exactly and leaves the codes alone
    q2, s2 = orc.quant_act((x.astype(np.float32) * 0.5).astype(np.float16))
    assert np.array_equal(q2, q) and np.array_equal(s2, s * np.float32(0.5))
    # a token's result does not depend on the other tokens in the batch
    q1, s1 = orc.quant_act(x[3:4])
    assert np.array_equal(q1[0], q[3]) and np.array_equal(s1[0], s[3])
    # negation flips the codes
    qn, sn = orc.quant_act(-x)
    assert np.array_equal(qn, -q) and np.array_equal(sn, s)


def test_quant_act_zero_group_and_exact_grid():
    x = np.zeros((2, 256), dtype=np.float16)
    c = np.random.default_rng(3).integers(-7, 8, size=128)
    c[5] = 7
    x[1, 128:] = (c * 0.25).astype(np.float16)          # s = 1.75/7 = 0.25 exactly
    q, s = orc.quant_act(x)
    assert not q[0].any() and not s[0].any() and s[1, 0] == 0
    assert s[1, 1] == np.float32(0.25)
    assert q[1, 128:].tolist() == c.tolist()


# ================================================================ O3 partials
def test_partials_vs_python_integers():
    M, N, K = 3, 5, 256
    rng = np.random.default_rng(9)
    qa = rng.integers(-7, 8, size=(M, K), dtype=np.int8)
    qw = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    P = orc.partials(qa, qw)
    assert P.shape == (M, N, 2) and P.dtype == np.int32
    for m in range(M):
        for n in range(N):
            for j in range(2):
                want = sum(int(qa[m, k]) * int(qw[n, k]) for k in range(128 * j, 128 * j + 128))
                assert int(P[m, n, j]) == want


def test_partials_bounds_and_sum():
    M, N, K = 4, 32, 1024
    rng = np.random.default_rng(10)
    qa = rng.integers(-7, 8, size=(M, K), dtype=np.int8)
    qw = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    qa[0, :128] = -7
    qw[0, :128] = -8                                     # the extreme group
    P = orc.partials(qa, qw)
    assert int(P[0, 0, 0]) == 128 * 56 == 7168
    assert np.abs(P).max() <= 7168
    full = qa.astype(np.int64) @ qw.astype(np.int64).T
    assert np.array_equal(P.sum(axis=2, dtype=np.int64), full)


# ================================================================ O4 W4A4 output
def _exact_w4a4(qa, sa, qw, sw, m, n):
    tot = Fraction(0)
    for k in range(qa.shape[1]):
        j = k // 128
        tot += (int(qa[m, k]) * F(sa[m, j])) * (int(qw[n, k]) * F(sw[n, j]))
    return tot


def test_gemm_w4a4_vs_exact_dequantise_then_matmul():
    M, N, K = 3, 6, 256
    codes, scales, x = synth.generic_case(21, M, N, K)
    qa, sa = orc.quant_act(x)
    y = orc.gemm_w4a4(qa, sa, codes, scales)
    assert y.shape == (M, N) and y.dtype == np.float16
    for m in range(M):
        for n in range(N):
            assert F(y[m, n]) == fl16(_exact_w4a4(qa, sa, codes, scales, m, n)), (m, n)


def test_gemm_w4a4_equals_float64_dequant_matmul():
    M, N, K = 5, 48, 1024
    codes, scales, x = synth.generic_case(22, M, N, K)
    qa, sa = orc.quant_act(x)
    G = K // 128
    a = qa.astype(np.float64) * np.repeat(sa.astype(np.float64), 128, axis=1)
    w = codes.astype(np.float64) * np.repeat(scales.astype(np.float64), 128, axis=1)
    ref = a @ w.T
    # also the stated invariant: y = sum_j P * sa * sw
    P = orc.partials(qa, codes).astype(np.float64)
    inv = np.zeros((M, N))
    for j in range(G):
        inv += P[:, :, j] * sa[:, j].astype(np.float64)[:, None] * scales[:, j].astype(np.float64)[None, :]
    assert np.allclose(ref, inv, rtol=1e-12, atol=1e-12)
    y = orc.gemm_w4a4(qa, sa, codes, scales).astype(np.float64)
    assert np.max(np.abs(y - ref)) <= np.max(np.abs(ref)) * 2.0 ** -11


def test_gemm_w4a4_unit_scales_is_integer_matmul():
    M, N, K = 4, 24, 256
    rng = np.random.default_rng(23)
    qa = rng.integers(-2, 3, size=(M, K), dtype=np.int8)
    qw = rng.integers(-2, 3, size=(N, K), dtype=np.int8)
    sa = np.ones((M, 2), np.float32)
    sw = np.ones((N, 2), np.float16)
    y = orc.gemm_w4a4(qa, sa, qw, sw)
    want = qa.astype(np.int64) @ qw.astype(np.int64).T
    assert np.abs(want).max() <= 2048
    assert np.array_equal(y.astype(np.int64), want)


# ================================================================ O5 W4A16 output
def test_gemm_w4a16_vs_exact_rationals():
    M, N, K = 3, 5, 256
    codes, scales, x = synth.generic_case(31, M, N, K)
    y = orc.gemm_w4a16(x, codes, scales)
    assert y.shape == (M, N) and y.dtype == np.float16
    for m in range(M):
        for n in range(N):
            tot = Fraction(0)
            for k in range(K):
                tot += F(x[m, k]) * int(codes[n, k]) * F(scales[n, k // 128])
            assert F(y[m, n]) == fl16(tot), (m, n)


def test_gemm_w4a16_exactly_representable_case():
    """Small integer x, power-of-two scales: every partial sum is an integer
    multiple of 2^-6 below 2^11, so the fp16 result is exact and unique."""
    M, N, K = 4, 16, 256
    rng = np.random.default_rng(32)
    x = rng.integers(-2, 3, size=(M, K)).astype(np.float16)
    qw = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    sw = np.tile(np.array([[2.0 ** -6, 2.0 ** -5]], np.float16), (N, 1))
    y = orc.gemm_w4a16(x, qw, sw).astype(np.float64)
    want = np.zeros((M, N))
    for j in range(2):
        blk = slice(128 * j, 128 * j + 128)
        want += (x[:, blk].astype(np.int64) @ qw[:, blk].astype(np.int64).T) * float(sw[0, j])
    assert np.array_equal(y, want)


def test_gemm_w4a16_linearity_and_column_locality():
    M, N, K = 4, 32, 512
    codes, scales, x = synth.generic_case(33, M, N, K)
    y = orc.gemm_w4a16(x, codes, scales)
    # column n depends on row n of the weight only
    codes2 = codes.copy()
    codes2[7] = -codes2[7].clip(-7, 7)
    y2 = orc.gemm_w4a16(x, codes2, scales)
    keep = np.arange(N) != 7
    assert np.array_equal(y[:, keep], y2[:, keep])
    assert not np.array_equal(y[:, 7], y2[:, 7])
    # row m depends on token m only; x -> 2x doubles y exactly (no overflow here)
    y3 = orc.gemm_w4a16((x.astype(np.float32) * 2).astype(np.float16), codes, scales)
    assert np.array_equal(y3, (y.astype(np.float32) * 2).astype(np.float16))
    assert np.array_equal(orc.gemm_w4a16(x[1:2], codes, scales)[0], y[1])
    # the sampled-column helper is the same product
    cols = np.array([3, 30, 7])
    assert np.array_equal(orc.gemm_w4a16_columns(x, codes, scales, cols), y[:, cols])


def test_w4a4_column_helper_is_the_column_slice_of_the_full_product():
    """gemm_w4a4_columns (the checker of full-size draft-mode outputs) against the columns of
    gemm_w4a4, itself pinned to exact rationals above: unsorted columns without repeats, a
    single column, all columns; independently, against a per-element integer/Fraction sum."""
    from fractions import Fraction
    M, N, K = 5, 48, 384
    codes, scales, x = synth.generic_case(36, M, N, K)
    qa, sa = orc.quant_act(x)
    y = orc.gemm_w4a4(qa, sa, codes, scales)
    for cols in (np.array([41, 3, 30, 7, 0, 47]), np.array([17]), np.arange(N)):
        got = orc.gemm_w4a4_columns(qa, sa, codes, scales, cols)
        assert got.dtype == np.float16 and got.shape == (M, len(cols))
        assert np.array_equal(got.view(np.uint16), y[:, cols].view(np.uint16))
    cols = np.array([41, 3, 30])
    got = orc.gemm_w4a4_columns(qa, sa, codes, scales, cols)
    for m in range(M):
        for c, n in enumerate(cols):
            acc = Fraction(0)
            for j in range(K // 128):
                P = sum(int(qa[m, k]) * int(codes[n, k]) for k in range(128 * j, 128 * j + 128))
                acc += P * Fraction(float(sa[m, j])) * Fraction(float(scales[n, j]))
            assert got[m, c] == np.float16(float(acc)) or abs(float(got[m, c]) - float(acc)) <= 2.0 ** -11 * abs(float(acc))


def test_planted_mistakes_in_the_column_helpers_fail_their_pin(monkeypatch):
    """A column helper that slices only the codes (scales of the first columns), or that
    sorts its columns, is caught."""
    def scales_not_sliced(qa, sa, qw, sw, cols, group=128):
        cols = np.asarray(cols)
        return orc.gemm_w4a4(qa, sa, np.asarray(qw)[cols], np.asarray(sw)[:len(cols)], group)

    def sorted_columns(qa, sa, qw, sw, cols, group=128):
        cols = np.sort(np.asarray(cols))
        return orc.gemm_w4a4(qa, sa, np.asarray(qw)[cols], np.asarray(sw)[cols], group)

    for mutant in (scales_not_sliced, sorted_columns):
        with monkeypatch.context() as mp:
            mp.setattr(orc, "gemm_w4a4_columns", mutant)
            with pytest.raises(AssertionError):
                test_w4a4_column_helper_is_the_column_slice_of_the_full_product()


def test_fp16_weight_rounding_variant_is_close_but_distinct():
    M, N, K = 8, 64, 1024
    codes, scales, x = synth.generic_case(34, M, N, K)
    ya = orc.gemm_w4a16(x, codes, scales).astype(np.float64)
    yb = orc.gemm_w4a16(x, codes, scales, round_weights_to_fp16=True).astype(np.float64)
    rel = np.max(np.abs(ya - yb)) / np.max(np.abs(ya))
    assert rel <= 2e-3


# ================================================================ cross-mode bound
def test_cross_mode_error_bound():
    """|y_w4a4 - y_w4a16| is bounded by what half a quantisation step per
    activation can do: sum_j sa/2 * sum_{k in j} |w[n,k]|."""
    M, N, K = 6, 40, 512
    codes, scales, x = synth.generic_case(41, M, N, K)
    qa, sa = orc.quant_act(x)
    y4 = orc.gemm_w4a4(qa, sa, codes, scales).astype(np.float64)
    y16 = orc.gemm_w4a16(x, codes, scales).astype(np.float64)
    w = np.abs(orc.dequant_weights(codes, scales)).reshape(N, K // 128, 128).sum(axis=2)   # [N, G]
    bound = 0.5 * (1 + 2.0 ** -20) * sa.astype(np.float64) @ w.T
    slack = 2.0 ** -9 * (np.abs(y4) + np.abs(y16))
    assert np.all(np.abs(y4 - y16) <= bound + slack)
    assert np.max(np.abs(y4 - y16)) > 0                    # the modes do differ


# ================================================================ input recipe
def test_synth_recipe_is_seeded_and_shaped():
    cfg = synth.CONFIGS[2]
    assert (cfg.draft_M, cfg.verify_M) == (8, 32)
    assert synth.CONFIGS[4].verify_M == 384 and synth.CONFIGS[5].verify_M == 512
    c1 = synth.weight_codes(2, 1, 64, 256)
    c2 = synth.weight_codes(2, 1, 64, 256)
    assert np.array_equal(c1, c2) and c1.min() == -8 and c1.max() == 7
    s = synth.weight_scales(2, 1, 64, 256)
    assert s.dtype == np.float16 and s.min() >= 0.002 and s.max() <= 0.01
    x = synth.activations(2, 1, 8, 4096, verify=False)
    ch = synth.outlier_channels(2, 1, 4096)
    assert len(ch) == 41 and x.dtype == np.float16
    assert np.abs(x[:, ch].astype(np.float32)).mean() > 10
    assert len(synth.outlier_channels(1, 0, 1024)) == 4


# ================================================================ acceptance policy and KV overwrite (Sec. 3.1)
from oracle import accept_oracle as acc   # noqa: E402


def _read_kv_fixture(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split(":", 1)
        out[k.strip()] = [int(t) for t in v.split()]
    return out


def _logits_with_top1(top, V, rng, dtype=np.float16):
    """[rows, V] random logits whose strict maximum in row j sits at top[j]."""
    lg = rng.standard_normal((len(top), V)).astype(np.float32)
    for j, t in enumerate(top):
        lg[j, t] = lg[j].max() + 1.0
    return lg.astype(dtype)


def test_accept_paper_mini_sample():
    """The worked example the paper gives for gamma = 4 (tests/golden/accept_minisample.txt)."""
    fx = _read_kv_fixture("accept_minisample.txt")
    gamma = fx["gamma"][0]
    rng = np.random.default_rng(5)
    emitted = 0
    for c in ("cycle1", "cycle2"):
        lg = _logits_with_top1(fx[f"{c}_verify_top1"], 128, rng)[None]
        a, out = acc.greedy_accept(lg, np.array([fx[f"{c}_draft"]], dtype=np.int32))
        assert a.tolist() == fx[f"{c}_accepted"]
        assert out[0].tolist() == fx[f"{c}_out"]
        emitted += int(a[0]) + 1
    assert gamma == 4 and emitted == fx["tokens_after_two_cycles"][0] == 8   # "commences from the ninth token"


def test_accept_equals_longest_common_prefix_formulation():
    """Independent formulation with library routines: a = length of the longest common
    prefix of the drafts and the verify pass's greedy tokens (np.argmax returns the first
    maximum); the emitted token is the greedy token at position a."""
    rng = np.random.default_rng(11)
    for V, gamma, B in [(3, 3, 64), (5, 5, 64), (17, 1, 32), (2, 4, 64)]:
        lg = rng.integers(-3, 4, (B, gamma + 1, V)).astype(np.float16)      # many ties and many matches
        draft = rng.integers(0, V, (B, gamma)).astype(np.int32)
        a, out = acc.greedy_accept(lg, draft)
        greedy = np.argmax(lg.astype(np.float64), axis=2)
        eq = (greedy[:, :gamma] == draft).astype(np.int64)
        a_ref = np.cumprod(eq, axis=1).sum(axis=1)
        assert a.tolist() == a_ref.tolist()
        for b in range(B):
            n = int(a[b])
            assert out[b, :n].tolist() == draft[b, :n].tolist()
            assert out[b, n] == greedy[b, n]
            assert (out[b, n + 1:] == -1).all()
            if n < gamma:
                assert out[b, n] != draft[b, n]          # a rejected draft is never what gets emitted


def test_accept_brute_force_all_small_cases():
    """Every combination of greedy tokens and drafts for V = 3, gamma = 2."""
    V, gamma = 3, 2
    import itertools
    for greedy in itertools.product(range(V), repeat=gamma + 1):
        lg = np.full((1, gamma + 1, V), -1.0, dtype=np.float16)
        for j, t in enumerate(greedy):
            lg[0, j, t] = 2.0
        for draft in itertools.product(range(V), repeat=gamma):
            a, out = acc.greedy_accept(lg, np.array([draft], dtype=np.int32))
            if draft[0] != greedy[0]:
                exp_a, exp_out = 0, [greedy[0], -1, -1]
            elif draft[1] != greedy[1]:
                exp_a, exp_out = 1, [draft[0], greedy[1], -1]
            else:
                exp_a, exp_out = 2, [draft[0], draft[1], greedy[2]]
            assert int(a[0]) == exp_a and out[0].tolist() == exp_out


def test_accept_ties_take_the_lowest_token_id_and_infinities_are_ordered():
    lg = np.zeros((1, 2, 6), dtype=np.float16)
    lg[0, 0, [2, 4]] = 3.0                       # tie between 2 and 4 -> 2
    lg[0, 1, :] = -np.inf
    lg[0, 1, 5] = -60000.0                       # the only finite value wins over -inf
    a, out = acc.greedy_accept(lg, np.array([[4]], dtype=np.int32))
    assert a.tolist() == [0] and out.tolist() == [[2, -1]]
    a, out = acc.greedy_accept(lg, np.array([[2]], dtype=np.int32))
    assert a.tolist() == [1] and out.tolist() == [[2, 5]]
    assert acc.top1(np.array([-np.inf, -np.inf])) == 0
    assert acc.top1(np.array([1.0, np.inf, np.inf])) == 1
    assert acc.top1(np.array([-0.0, 0.0])) == 0          # -0 and +0 compare equal: a tie


def test_accept_rows_are_independent():
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((6, 4, 50)).astype(np.float16)
    draft = np.argmax(lg[:, :3], axis=2).astype(np.int32)
    draft[::2, 1] = (draft[::2, 1] + 1) % 50             # reject the second draft of every other sequence
    a, out = acc.greedy_accept(lg, draft)
    assert a.tolist() == [1, 3, 1, 3, 1, 3]
    for b in range(6):
        a1, out1 = acc.greedy_accept(lg[b:b + 1], draft[b:b + 1])
        assert a1[0] == a[b] and out1[0].tolist() == out[b].tolist()


def test_kv_overwrite_touches_exactly_the_accepted_rows():
    rng = np.random.default_rng(9)
    B, S, D, gamma = 4, 12, 8, 3
    cache = rng.standard_normal((B, S, D)).astype(np.float16)
    kv = rng.standard_normal((B, gamma + 1, D)).astype(np.float16)
    a = np.array([0, 3, 1, 2], dtype=np.int32)
    pos = np.array([5, 0, 10, 11], dtype=np.int32)       # the last one runs off the end of the cache
    new = acc.kv_overwrite(cache, kv, a, pos)
    for b in range(B):
        for s in range(S):
            j = s - int(pos[b])
            if 0 <= j <= int(a[b]):
                assert (new[b, s] == kv[b, j]).all()
            else:
                assert (new[b, s] == cache[b, s]).all()
    assert (cache != new).any()                          # the input itself is not modified ...
    assert acc.kv_overwrite(new, kv, a, pos).tobytes() == new.tobytes()   # ... and the step is idempotent


# ---------------------------------------------------------------- producers of draft-mode activations
from oracle import producers_oracle as prod


def _f16(values):
    return np.asarray(values, dtype=np.float16)


def _exact_rsqrt_fp32(v: Fraction) -> Fraction:
    """fp32(1/sqrt(v)) for a positive rational v, by integer square root at 2^-200."""
    import math
    scale = 1 << 400
    root = Fraction(math.isqrt((v.numerator * scale) // v.denominator), 1 << 200)   # sqrt(v), 200 bits
    return _fl(1 / root, 23, -126)


def test_rmsnorm_vs_exact_rationals():
    rng = np.random.default_rng(41)
    K = 128
    x = _f16(rng.standard_normal((3, K)) * 2.0)
    w = _f16(1.0 + 0.25 * rng.standard_normal(K))
    eps = np.float32(1e-5)
    got = prod.rmsnorm_f16(x, w, eps)
    for m in range(3):
        ms = sum(Fraction(float(v)) ** 2 for v in x[m]) / K
        r = _exact_rsqrt_fp32(ms + Fraction(float(eps)))
        for k in range(K):
            u = _fl(Fraction(float(x[m, k])) * Fraction(float(w[k])) * r, 23, -126)
            h = _fl(u, 10, -14)
            assert Fraction(float(got[m, k])) == h, (m, k)


def test_rmsnorm_closed_forms():
    K = 4096
    ones = _f16(np.ones(K))
    # constant row, eps = 0: every output is sign(c) * w
    for c in (0.37, -3.0, 1024.0):
        h = prod.rmsnorm_f16(_f16(np.full((1, K), c)), ones, 0.0)
        assert np.all(h == np.float16(np.sign(c)))
    w = _f16(np.linspace(0.5, 1.5, K))
    h = prod.rmsnorm_f16(_f16(np.full((1, K), 2.0)), w, 0.0)
    assert np.array_equal(h[0], w)                      # the weight multiplies, per feature
    # one-hot row: mean square v^2/K, so the live output is sign(v) * sqrt(K) * w_k
    x = np.zeros((1, K), dtype=np.float16)
    x[0, 77] = -0.5
    h = prod.rmsnorm_f16(x, w, 0.0)
    assert h[0, 77] == np.float16(-64.0 * np.float32(w[77])) and np.count_nonzero(h) == 1
    # eps sits inside the square root, added to the MEAN of squares: c = 2, eps = 12 -> 1/sqrt(16)
    h = prod.rmsnorm_f16(_f16(np.full((1, K), 2.0)), ones, 12.0)
    assert np.all(h == np.float16(0.5))
    # a zero row stays zero (no 0/0) once eps > 0
    assert not np.any(prod.rmsnorm_f16(np.zeros((2, K), np.float16), w, 1e-6))


def test_rmsnorm_scale_invariance_and_row_independence():
    rng = np.random.default_rng(42)
    x = _f16(rng.standard_normal((4, 512)))
    w = _f16(1.0 + 0.1 * rng.standard_normal(512))
    a = prod.rmsnorm_f16(x, w, 0.0)
    b = prod.rmsnorm_f16(_f16(x.astype(np.float32) * 4.0), w, 0.0)     # exact scaling by a power of two
    assert np.array_equal(a, b)
    x2 = x.copy()
    x2[2] = _f16(rng.standard_normal(512) * 9.0)
    c = prod.rmsnorm_f16(x2, w, 0.0)
    assert np.array_equal(a[[0, 1, 3]], c[[0, 1, 3]]) and not np.array_equal(a[2], c[2])


def test_rmsnorm_vs_torch_cpu_float64():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(43)
    x = _f16(rng.standard_normal((5, 1024)) * 3.0)
    w = _f16(1.0 + 0.2 * rng.standard_normal(1024))
    eps = 1e-5
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x.astype(np.float64)), (1024,),
                                       torch.from_numpy(w.astype(np.float64)), float(np.float32(eps))).numpy()
    got = prod.rmsnorm_f16(x, w, eps).astype(np.float64)
    # the oracle rounds twice (binary32, then fp16): at most one fp16 ulp from the real value, mostly exact
    ulp = np.maximum(np.abs(ref), 2.0 ** -14) * 2.0 ** -10
    assert np.all(np.abs(got - ref) <= 0.5001 * ulp + 1e-12)
    assert np.mean(got == ref.astype(np.float16).astype(np.float64)) > 0.999


def test_silu_mul_vs_high_precision_decimal():
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    gs = [0.0, 0.5, -0.5, 1.0986328125, -3.25, 7.0, -11.0, 20.0, -20.0, 60.0, 0.0001220703125, -65504.0]
    us = [1.5, -2.25, 0.33349609375, 1.0, -7.0, 0.125, 3.0, -1.0, 2.0, 0.5, 1000.0, 1.0]
    gu = _f16([gs + us])
    got = prod.silu_mul_f16(gu)[0]
    for i, (g, u) in enumerate(zip(gu[0, :len(gs)], gu[0, len(gs):])):
        gd = Decimal(float(g))
        s_exact = Fraction(gd / (1 + (-gd).exp())) if float(g) > -1000 else Fraction(0)
        s32 = _fl(s_exact, 23, -126)
        t32 = _fl(s32 * Fraction(float(u)), 23, -126)
        assert Fraction(float(got[i])) == _fl(t32, 10, -14), (i, float(g), float(u))


def test_silu_mul_closed_forms_and_column_order():
    I = 256
    rng = np.random.default_rng(44)
    up = _f16(rng.standard_normal(I) * 2.0)
    gate = _f16(rng.standard_normal(I) * 3.0)
    # SiLU(0) = 0 whatever up holds
    assert not np.any(prod.silu_mul_f16(np.concatenate([np.zeros(I, np.float16), up])[None, :]))
    # large gate: SiLU is the identity in binary32, so h = fp16(g * u); gate is the FIRST half
    big = _f16(np.full(I, 32.0))
    h = prod.silu_mul_f16(np.concatenate([big, up])[None, :])[0]
    assert np.array_equal(h, (np.float32(32.0) * up.astype(np.float32)).astype(np.float16))
    h_swapped = prod.silu_mul_f16(np.concatenate([up, big])[None, :])[0]
    assert not np.array_equal(h, h_swapped)
    # SiLU(ln 3) = 0.75 ln 3 (sigmoid(ln 3) = 3/4), here through a gate that is fp16(ln 3)
    g = np.float16(np.log(3.0))
    sig = 1.0 / (1.0 + np.exp(-np.float64(g)))
    h = prod.silu_mul_f16(_f16([[g, 1.0]]))[0, 0]
    assert h == np.float16(np.float32(np.float64(g) * sig)) and abs(float(h) - 0.75 * np.log(3.0)) < 1e-3
    # SiLU(g) - SiLU(-g) = g, to binary32 accuracy before the fp16 rounding: with up = 1 the two
    # fp16 results differ by g within one fp16 ulp of the larger
    ones = np.ones(I, np.float16)
    p = prod.silu_mul_f16(np.concatenate([gate, ones])[None, :])[0].astype(np.float64)
    n = prod.silu_mul_f16(np.concatenate([-gate, ones])[None, :])[0].astype(np.float64)
    assert np.all(np.abs((p - n) - gate.astype(np.float64)) <= np.maximum(np.abs(p), np.abs(n)) * 2.0 ** -10 + 1e-7)


def test_silu_mul_vs_torch_cpu_float64():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(45)
    gu = _f16(rng.standard_normal((3, 2 * 384)) * 2.5)
    g = torch.from_numpy(gu[:, :384].astype(np.float64))
    u = torch.from_numpy(gu[:, 384:].astype(np.float64))
    ref = (torch.nn.functional.silu(g) * u).numpy()
    got = prod.silu_mul_f16(gu).astype(np.float64)
    ulp = np.maximum(np.abs(ref), 2.0 ** -14) * 2.0 ** -10
    assert np.all(np.abs(got - ref) <= 0.5001 * ulp + 1e-12)
    assert np.mean(got == ref.astype(np.float16).astype(np.float64)) > 0.999


# ---------------------------------------------------------------- rotation in front of the quantiser
from oracle import rotation_oracle as rot


def _h128():
    from scipy.linalg import hadamard
    return hadamard(128).astype(np.float64)


def test_hadamard_equals_the_matrix_product_where_sums_are_exact():
    rng = np.random.default_rng(51)
    x = rng.integers(-40, 41, size=(5, 384)).astype(np.float16)          # small integers: every partial sum is exact
    x[4] *= np.float16(0.25)                                             # and a row of quarter-integers
    got = rot.hadamard128_f16(x)
    ref = (x.astype(np.float64).reshape(5, 3, 128) @ _h128() / 8.0).reshape(5, 384)
    assert np.array_equal(got.astype(np.float64), ref.astype(np.float16).astype(np.float64))
    assert np.abs(ref).max() > 100                                       # not a trivial case


def test_hadamard_entries_on_one_hot_rows():
    x = np.zeros((128, 128), dtype=np.float16)
    x[np.arange(128), np.arange(128)] = 8.0
    got = rot.hadamard128_f16(x).astype(np.int64)
    for i in (0, 1, 2, 3, 64, 85, 127):
        for j in range(128):
            assert got[i, j] == (-1) ** bin(i & j).count("1")
    assert np.array_equal(got, got.T) and np.array_equal(got @ got.T, 128 * np.eye(128, dtype=np.int64))


def test_hadamard_groups_are_independent_and_twice_is_doubling():
    rng = np.random.default_rng(52)
    x = rng.integers(-6, 7, size=(3, 256)).astype(np.float16)
    once = rot.hadamard128_f16(x)
    twice = rot.hadamard128_f16(once)                                    # (1/8)(1/8) H H = 2 I, exact on these inputs
    assert np.array_equal(twice.astype(np.float32), 2.0 * x.astype(np.float32))
    x2 = x.copy()
    x2[:, 128:] = rng.integers(-6, 7, size=(3, 128)).astype(np.float16)
    assert np.array_equal(rot.hadamard128_f16(x2)[:, :128], once[:, :128])


def test_hadamard_general_inputs_close_to_float64_and_energy_kept():
    rng = np.random.default_rng(53)
    x = (rng.standard_normal((4, 512)) * 3.0).astype(np.float16)
    x[:, 7] *= 20
    got = rot.hadamard128_f16(x).astype(np.float64)
    ref = (x.astype(np.float64).reshape(4, 4, 128) @ _h128() / 8.0).reshape(4, 512)
    assert np.all(np.abs(got - ref) <= np.maximum(np.abs(ref), 1e-3) * 2.0 ** -10)
    e_in = (x.astype(np.float64) ** 2).reshape(4, 4, 128).sum(-1)
    e_out = (got ** 2).reshape(4, 4, 128).sum(-1)
    assert np.allclose(e_out, 2.0 * e_in, rtol=2e-3)                     # |x H / 8|^2 = 128 / 64 |x|^2


def test_rotation_lowers_the_draft_mode_error_on_outlier_channels():
    """The purpose of the rotation: with one channel in a hundred 20 times larger, the
    4-bit activation grid of its group is 20 times coarser for the other 127 channels;
    after the rotation the energy is spread.  Weights are the same random codes in both
    runs (they stand for a checkpoint quantised in the respective basis)."""
    codes, scales, x = synth.generic_case(54, 16, 64, 1024)
    w = orc.dequant_weights(codes, scales) if hasattr(orc, "dequant_weights") else \
        codes.astype(np.float64) * np.repeat(scales.astype(np.float64), 128, axis=1)

    def rel_err(xin):
        qa, sa = orc.quant_act(xin)
        xq = qa.astype(np.float64) * np.repeat(sa.astype(np.float64), 128, axis=1)
        exact = xin.astype(np.float64) @ w.T
        return np.linalg.norm(xq @ w.T - exact) / np.linalg.norm(exact)

    plain, rotated = rel_err(x), rel_err(rot.hadamard128_f16(x))
    assert rotated < 0.6 * plain, (plain, rotated)


# ---------------------------------------------------------------- reordering quantiser (outlier groups at ~8 bits)
from oracle import reorder_oracle as reo


def test_reorder_quant_hand_worked_group():
    rows = {}
    for line in open(os.path.join(GOLDEN, "reorder_quant_worked_group.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        key, vals = line.split(":")
        rows[key.strip()] = [float(v) for v in vals.split()]
    x = np.zeros((1, 128), dtype=np.float16)
    x[0, :8] = rows["x"]
    codes, scales = reo.reorder_quant(x, np.arange(128), 1)
    assert codes.shape == (1, 256) and scales.shape == (1, 2)
    assert codes[0, :8].tolist() == rows["hi"] and codes[0, 128:136].tolist() == rows["lo"]
    assert not codes[0, 8:128].any() and not codes[0, 136:].any()
    assert scales[0].tolist() == [rows["scale_hi"][0], rows["scale_lo"][0]]


def test_reorder_quant_digits_cover_the_whole_range():
    for q8 in range(-119, 120):
        lo = ((q8 + 8) % 16) - 8
        hi = (q8 - lo) // 16
        assert -8 <= lo <= 7 and -7 <= hi <= 7 and 16 * hi + lo == q8
    # through the oracle: a group holding every level once (a = 119, s = 1)
    x = np.zeros((1, 256), dtype=np.float16)
    x[0, :239] = np.arange(-119, 120)
    perm = np.concatenate([np.arange(128, 256), np.arange(0, 128)])      # put group 0 last, as the outlier group
    codes, scales = reo.reorder_quant(x, perm, 1)
    hi, lo = codes[0, 128:256].astype(np.int64), codes[0, 256:384].astype(np.int64)
    assert np.array_equal(16 * hi + lo, np.arange(-119, 9))              # the gathered group 0 of x
    assert scales[0, 1] == 16.0 and scales[0, 2] == 1.0


def test_reorder_quant_vs_exact_rationals():
    rng = np.random.default_rng(61)
    K, Go = 384, 2
    x = (rng.standard_normal((3, K)) * 2.0).astype(np.float16)
    x[:, [5, 130, 300]] *= 20
    perm = rng.permutation(K)
    codes, scales = reo.reorder_quant(x, perm, Go)
    G = K // 128
    for m in range(3):
        for g in range(G):
            vals = [Fraction(float(x[m, perm[g * 128 + i]])) for i in range(128)]
            a = max(abs(v) for v in vals)
            if g < G - Go:
                s = _fl(a / 7, 23, -126)
                q = [max(-8, min(7, _round_half_even(_fl(v / s, 23, -126)))) for v in vals]
                assert codes[m, g * 128:(g + 1) * 128].tolist() == q
                assert Fraction(float(scales[m, g])) == s
            else:
                s = _fl(a / 119, 23, -126)
                q8 = [max(-119, min(119, _round_half_even(_fl(v / s, 23, -126)))) for v in vals]
                o = (G - Go + 2 * (g - (G - Go))) * 128
                hi = codes[m, o:o + 128].astype(np.int64)
                lo = codes[m, o + 128:o + 256].astype(np.int64)
                assert (16 * hi + lo).tolist() == q8 and lo.min() >= -8 and lo.max() <= 7 and abs(hi).max() <= 7
                assert Fraction(float(scales[m, o // 128])) == 16 * s and Fraction(float(scales[m, o // 128 + 1])) == s


def test_reorder_quant_ordinary_groups_equal_the_plain_quantiser_on_the_gathered_tensor():
    rng = np.random.default_rng(62)
    x = rng.standard_normal((4, 512)).astype(np.float16)
    perm = rng.permutation(512)
    codes, scales = reo.reorder_quant(x, perm, 1)
    q_ref, s_ref = orc.quant_act(np.ascontiguousarray(x[:, perm]))
    assert np.array_equal(codes[:, :384], q_ref[:, :384]) and np.array_equal(scales[:, :3], s_ref[:, :3])
    c0, s0 = reo.reorder_quant(x, perm, 0)                               # no outlier group: the plain quantiser
    assert np.array_equal(c0, q_ref) and np.array_equal(s0, s_ref)
    x[2] = 0
    codes, scales = reo.reorder_quant(x, perm, 2)
    assert not codes[2].any() and not scales[2].any()                    # zero row: zero scales, zero codes


def test_reorder_quant_product_identity_with_duplicated_weight_groups():
    """Integer check: with s = 1 in every group the draft-mode sum over the expanded
    dimension equals the plain integer product of the 8-bit / 4-bit codes."""
    rng = np.random.default_rng(63)
    K, Go, N = 384, 1, 8
    perm = rng.permutation(K)
    x = np.zeros((2, K), dtype=np.float16)
    xr = rng.integers(-7, 8, (2, K)).astype(np.float16)
    xr[:, :256][:, [0, 128]] = 7                                         # a = 7 in the ordinary groups -> s = 1
    xr[:, 256:] = rng.integers(-119, 120, (2, 128))
    xr[:, 256] = 119                                                     # a = 119 in the outlier group -> s = 1
    x[:, perm] = xr
    w = rng.integers(-8, 8, (N, K))
    codes, scales = reo.reorder_quant(x, perm, Go)
    wx = reo.expand_weight_columns(w, perm, Go)
    assert wx.shape == (N, K + 128)
    deq = codes.astype(np.int64) * np.repeat(scales.astype(np.int64), 128, axis=1)
    assert np.array_equal(deq @ wx.T, xr.astype(np.int64) @ w[:, perm].T)


def test_reordering_lowers_the_draft_mode_error_on_outlier_channels():
    codes, scales, x = synth.generic_case(55, 32, 256, 4096)
    w = codes.astype(np.float64) * np.repeat(scales.astype(np.float64), 128, axis=1)
    order = np.argsort(-np.abs(x.astype(np.float64)).mean(axis=0), kind="stable")
    perm = np.concatenate([np.sort(order[128:]), np.sort(order[:128])])  # the 128 largest channels last
    exact = x.astype(np.float64) @ w.T
    qa, sa = orc.quant_act(x)
    plain = np.linalg.norm((qa * np.repeat(sa.astype(np.float64), 128, axis=1)) @ w.T - exact) / np.linalg.norm(exact)
    qr, sr = reo.reorder_quant(x, perm, 1)
    wx = reo.expand_weight_columns(w, perm, 1)
    reordered = np.linalg.norm((qr * np.repeat(sr.astype(np.float64), 128, axis=1)) @ wx.T - exact) / np.linalg.norm(exact)
    assert reordered < 0.3 * plain, (plain, reordered)


# ---------------------------------------------------------------- the pins do bite
def _caught(monkeypatch, module, name, mutant, pins):
    """True if at least one of the pin tests fails once `module.name` is replaced by `mutant`."""
    with monkeypatch.context() as mp:
        mp.setattr(module, name, mutant)
        for pin in pins:
            try:
                pin()
            except AssertionError:
                return True
            except Exception:
                return True
    return False


def test_planted_mistakes_in_the_newer_oracles_fail_their_pins(monkeypatch):
    f32, f64, f16 = np.float32, np.float64, np.float16

    # ---- RMSNorm
    def rms_variant(eps_outside=False, mean_abs=False, drop_weight=False):
        def fn(x, w, eps):
            x64 = x.astype(f64)
            stat = np.mean(np.abs(x64), axis=1) ** 2 if mean_abs else np.sum(x64 * x64, axis=1) / x.shape[1]
            e = f64(f32(eps))
            r = (1.0 / (np.sqrt(stat) + e) if eps_outside else 1.0 / np.sqrt(stat + e)).astype(f32)
            t = x.astype(f32) * (1.0 if drop_weight else w.astype(f32)[None, :])
            return (t * r[:, None]).astype(f32).astype(f16)
        return fn
    rms_pins = [test_rmsnorm_vs_exact_rationals, test_rmsnorm_closed_forms, test_rmsnorm_vs_torch_cpu_float64]
    assert not _caught(monkeypatch, prod, "rmsnorm_f16", rms_variant(), rms_pins)          # the faithful copy passes
    for kw in (dict(eps_outside=True), dict(mean_abs=True), dict(drop_weight=True)):
        assert _caught(monkeypatch, prod, "rmsnorm_f16", rms_variant(**kw), rms_pins), kw

    # ---- SiLU * up
    def silu_variant(sign=-1.0, swap=False, sigmoid_only=False):
        def fn(gu):
            I = gu.shape[1] // 2
            g, u = (gu[:, I:], gu[:, :I]) if swap else (gu[:, :I], gu[:, I:])
            g = g.astype(f64)
            with np.errstate(over="ignore", invalid="ignore"):
                s = ((1.0 if sigmoid_only else g) / (1.0 + np.exp(sign * g))).astype(f32)
            return (s * u.astype(f32)).astype(f32).astype(f16)
        return fn
    silu_pins = [test_silu_mul_vs_high_precision_decimal, test_silu_mul_closed_forms_and_column_order,
                 test_silu_mul_vs_torch_cpu_float64]
    assert not _caught(monkeypatch, prod, "silu_mul_f16", silu_variant(), silu_pins)
    for kw in (dict(sign=1.0), dict(swap=True), dict(sigmoid_only=True)):
        assert _caught(monkeypatch, prod, "silu_mul_f16", silu_variant(**kw), silu_pins), kw

    # ---- rotation
    def had_variant(scale=0.125, reversed_difference=False, block=128):
        def fn(x):
            M, K = x.shape
            v = x.astype(f32).reshape(M, K // block, block)
            h = 1
            while h < block:
                p = v.reshape(M, K // block, block // (2 * h), 2, h)
                lo, hi = p[..., 0, :], p[..., 1, :]
                v = np.stack([lo + hi, (hi - lo) if reversed_difference else (lo - hi)], axis=-2)
                h *= 2
            return (v.reshape(M, K) * f32(scale)).astype(f16)
        return fn
    had_pins = [test_hadamard_equals_the_matrix_product_where_sums_are_exact, test_hadamard_entries_on_one_hot_rows,
                test_hadamard_groups_are_independent_and_twice_is_doubling]
    assert not _caught(monkeypatch, rot, "hadamard128_f16", had_variant(), had_pins)
    for kw in (dict(scale=1.0 / 16), dict(reversed_difference=True), dict(block=64)):
        assert _caught(monkeypatch, rot, "hadamard128_f16", had_variant(**kw), had_pins), kw

    # ---- reordering quantiser: planted through its constants and its digit split
    reo_pins = [test_reorder_quant_hand_worked_group, test_reorder_quant_vs_exact_rationals,
                test_reorder_quant_product_identity_with_duplicated_weight_groups]
    with monkeypatch.context() as mp:
        mp.setattr(reo, "LEVELS", 127)
        caught = False
        for pin in reo_pins:
            try:
                pin()
            except AssertionError:
                caught = True
                break
        assert caught
    original = reo.reorder_quant

    def swapped_digits(x, perm, Go):
        codes, scales = original(x, perm, Go)
        G = x.shape[1] // 128
        c = codes.reshape(x.shape[0], G + Go, 128).copy()
        for t in range(Go):
            a = G - Go + 2 * t
            c[:, [a, a + 1]] = c[:, [a + 1, a]]
        return c.reshape(codes.shape), scales
    assert _caught(monkeypatch, reo, "reorder_quant", swapped_digits, reo_pins)

    def inverse_permutation(x, perm, Go):
        return original(x, np.argsort(np.asarray(perm)), Go)
    assert _caught(monkeypatch, reo, "reorder_quant", inverse_permutation, reo_pins)
    assert not _caught(monkeypatch, reo, "reorder_quant", original, reo_pins)
