"""GPU-vs-oracle parity through the C ABI (run with -m gpu on an MI355X).

Integer stages (weight blob, activation codes and scales, per-group int32
partial sums) must match bit for bit; fp16 outputs must satisfy
max|y - y_ref| / max|y_ref| <= 2e-3 against the float64 oracle."""
import numpy as np
import pytest

from oracle import device_layout as lay
from oracle import qspec_oracle as orc
from paper_2410_11305_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2410_11305_amd import binding as B
    assert torch.cuda.is_available()
    B.lib()                                   # raises if the HIP library is missing
    return torch, B


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(y, ref):
    y = y.astype(np.float64)
    ref = ref.astype(np.float64)
    return float(np.max(np.abs(y - ref)) / max(np.max(np.abs(ref)), 1e-30))


SMALL_SHAPES = [(1, 128, 128), (3, 256, 256), (4, 1152, 1024), (5, 128, 1024), (16, 256, 128),
                (17, 1152, 256), (33, 144, 384), (70, 272, 640), (130, 48, 1280), (200, 80, 256),
                (40, 64, 128), (100, 32, 256), (65, 16, 128),
                (1100, 144, 256), (2050, 272, 384)]          # prefill-sized M: many ragged token blocks


# ------------------------------------------------------------------ pack
@pytest.mark.parametrize("N,K", [(16, 128), (48, 384), (1152, 1024), (4096, 11008)])
def test_pack_weights_byte_exact_and_roundtrip(env, N, K):
    torch, B = env
    codes, scales, _ = synth.generic_case(100 + N + K, 1, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    assert blob.numel() == B.packed_weight_bytes(N, K)
    assert np.array_equal(blob.cpu().numpy(), lay.weight_blob(codes, scales))
    c2, s2 = B.unpack_weights(blob, N, K)
    assert np.array_equal(c2.cpu().numpy(), codes)
    assert np.array_equal(s2.cpu().numpy().view(np.uint16), scales.view(np.uint16))


# ------------------------------------------------------------------ quant_act
def _check_quant(torch, B, x):
    q_ref, s_ref = orc.quant_act(x)
    qa, sa = B.quant_act(dev(torch, x))
    torch.cuda.synchronize()
    assert np.array_equal(sa.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(qa.cpu().numpy(), lay.act_bytes(q_ref))
    return qa, sa, q_ref, s_ref


@pytest.mark.parametrize("M,K", [(1, 128), (3, 256), (4, 1024), (5, 1024), (16, 128), (17, 256),
                                 (8, 4096), (32, 11008), (128, 28672)])
def test_quant_act_bit_exact(env, M, K):
    torch, B = env
    _, _, x = synth.generic_case(200 + M + K, M, 16, K)
    _check_quant(torch, B, x)


def test_quant_act_special_values(env):
    torch, B = env
    x = np.zeros((6, 256), dtype=np.float16)
    x[0, :8] = [7, -3.5, 0.5, 1.5, 2.5, -0.5, -2.5, 3.5]            # ties at scale 1
    x[1, 128:136] = [1.75, -0.875, 0.125, 0.375, 0.625, -0.125, -0.625, 0.875]   # ties at scale 0.25
    x[2, :4] = [65504, -65504, 32752, 4678]                         # fp16 extremes
    x[3, :4] = np.array([6e-8, 1.2e-7, -6e-8, 2.4e-7], np.float16)  # fp16 subnormals
    x[4, 128:] = np.linspace(-3, 3, 128).astype(np.float16)         # row 4 first group all zero
    x[5] = np.random.default_rng(1).standard_normal(256).astype(np.float16)
    qa, sa, q_ref, s_ref = _check_quant(torch, B, x)
    assert q_ref[0, :8].tolist() == [7, -4, 0, 2, 2, 0, -2, 4]
    assert s_ref[4, 0] == 0


def test_quant_act_all_fp16_magnitudes(env):
    """Every finite non-negative fp16 bit pattern as a value, against group
    maxima spread over the whole range."""
    torch, B = env
    vals = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16)      # 31744 values
    x = np.resize(vals, (248, 128)).copy()
    rng = np.random.default_rng(4)
    x *= rng.choice(np.array([1, -1], np.float16), size=x.shape)
    tops = np.resize(np.array([65504, 1000, 3.14, 0.007, 6.1e-5, 6e-8, 1.0, 21.0], np.float16), 248)
    x[:, 0] = np.maximum(np.abs(x).max(axis=1), tops)
    _check_quant(torch, B, x)


# ------------------------------------------------------------------ partials
@pytest.mark.parametrize("M,N,K", SMALL_SHAPES)
def test_partials_bit_exact(env, M, N, K):
    torch, B = env
    codes, scales, x = synth.generic_case(300 + M + N + K, M, N, K)
    q_ref, _ = orc.quant_act(x)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    qa = dev(torch, lay.act_bytes(q_ref))
    P = B.gemm_w4a4_partials(blob, qa, N, 0, N)
    assert np.array_equal(P.cpu().numpy(), orc.partials(q_ref, codes))
    if N >= 48:
        P2 = B.gemm_w4a4_partials(blob, qa, N, 16, 32)
        assert np.array_equal(P2.cpu().numpy(), orc.partials(q_ref, codes[16:48]))


def test_partials_extreme_codes(env):
    """All-(-8) weights against all-(+-7) activations: |P| reaches 128*56."""
    torch, B = env
    M, N, K = 16, 32, 256
    qw = np.full((N, K), -8, np.int8)
    qw[1::2] = 7
    q = np.full((M, K), -7, np.int8)
    q[::3] = 7
    sw = np.full((N, K // 128), 0.005, np.float16)
    blob = B.pack_weights(dev(torch, qw), dev(torch, sw))
    P = B.gemm_w4a4_partials(blob, dev(torch, lay.act_bytes(q)), N, 0, N).cpu().numpy()
    assert np.array_equal(P, orc.partials(q, qw))
    assert np.abs(P).max() == 7168


# ------------------------------------------------------------------ W4A4 output
@pytest.mark.parametrize("M,N,K", SMALL_SHAPES)
def test_gemm_w4a4_small(env, M, N, K):
    torch, B = env
    codes, scales, x = synth.generic_case(400 + M + N + K, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    qa, sa, q_ref, s_ref = _check_quant(torch, B, x)
    y = B.gemm_w4a4(blob, qa, sa, N).cpu().numpy()
    ref = orc.gemm_w4a4(q_ref, s_ref, codes, scales)
    assert rel_err(y, ref) <= TOL


def test_gemm_w4a4_unit_scales_bit_exact(env):
    """sa = sw = 1 and small codes: y is an integer below 2048, exact in fp16
    whatever the summation order."""
    torch, B = env
    M, N, K = 20, 64, 512
    rng = np.random.default_rng(5)
    q = rng.integers(-2, 3, size=(M, K), dtype=np.int8)
    qw = rng.integers(-2, 3, size=(N, K), dtype=np.int8)
    sw = np.ones((N, K // 128), np.float16)
    sa = np.ones((M, K // 128), np.float32)
    blob = B.pack_weights(dev(torch, qw), dev(torch, sw))
    y = B.gemm_w4a4(blob, dev(torch, lay.act_bytes(q)), dev(torch, sa), N).cpu().numpy()
    want = (q.astype(np.int64) @ qw.astype(np.int64).T)
    assert np.array_equal(y.astype(np.int64), want)
    assert np.array_equal(y, orc.gemm_w4a4(q, sa, qw, sw))


# ------------------------------------------------------------------ W4A16 output
@pytest.mark.parametrize("M,N,K", SMALL_SHAPES)
def test_gemm_w4a16_small(env, M, N, K):
    torch, B = env
    codes, scales, x = synth.generic_case(500 + M + N + K, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    y = B.gemm_w4a16(blob, dev(torch, x), N).cpu().numpy()
    ref = orc.gemm_w4a16(x, codes, scales)
    assert rel_err(y, ref) <= TOL


def test_gemm_w4a16_exactly_representable_bit_exact(env):
    torch, B = env
    M, N, K = 37, 96, 256
    rng = np.random.default_rng(6)
    x = rng.integers(-2, 3, size=(M, K)).astype(np.float16)
    qw = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    sw = np.tile(np.array([[2.0 ** -6, 2.0 ** -5]], np.float16), (N, 1))
    blob = B.pack_weights(dev(torch, qw), dev(torch, sw))
    y = B.gemm_w4a16(blob, dev(torch, x), N).cpu().numpy()
    assert np.array_equal(y, orc.gemm_w4a16(x, qw, sw))


def test_all_sixteen_codes_dequantise_exactly(env):
    """x = one-hot rows pick single weights: y[m, n] = code * scale exactly."""
    torch, B = env
    N, K = 16, 128
    qw = np.zeros((N, K), np.int8)
    for n in range(N):
        qw[n] = np.roll(np.arange(-8, 8, dtype=np.int8).repeat(8), n)
    sw = np.full((N, 1), 0.5, np.float16)
    x = np.eye(K, dtype=np.float16)                      # M = K = 128 one-hot tokens
    blob = B.pack_weights(dev(torch, qw), dev(torch, sw))
    y = B.gemm_w4a16(blob, dev(torch, x), N).cpu().numpy()
    assert np.array_equal(y, (qw.T.astype(np.float32) * 0.5).astype(np.float16))


# ------------------------------------------------------------------ tiled kernels (M > 32)
@pytest.mark.parametrize("S", [1, 3])
@pytest.mark.parametrize("shape", range(7))
def test_tile_kernels_every_workgroup_shape(env, plan, shape, S):
    """Every instantiated workgroup shape, alone and with 3 K-slices that meet in
    the workspace, on a problem with ragged M, a ragged last n-block and a group
    count (7) that does not divide by the slice count."""
    torch, B = env
    M, N, K = 150, 304, 896
    plan("QSPEC_TILE_W4A4", f"{shape % 4},{S}")      # 4 draft-mode shapes, 7 verify-mode shapes
    plan("QSPEC_TILE_W4A16", f"{shape},{S}")
    codes, scales, x = synth.generic_case(600 + shape, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    qa, sa, q_ref, s_ref = _check_quant(torch, B, x)
    need = B.workspace_bytes(M, N, K)
    assert (need > 0) == (S > 1)
    ws = B.alloc_workspace(need)
    ref4 = orc.gemm_w4a4(q_ref, s_ref, codes, scales)
    ref16 = orc.gemm_w4a16(x, codes, scales)
    xd = dev(torch, x)
    outs = []
    for _ in range(2):                      # the second call finds the counters as the first left them
        y4 = B.gemm_w4a4(blob, qa, sa, N, workspace=ws)
        y16 = B.gemm_w4a16(blob, xd, N, workspace=ws)
        torch.cuda.synchronize()
        assert rel_err(y4.cpu().numpy(), ref4) <= TOL
        assert rel_err(y16.cpu().numpy(), ref16) <= TOL
        outs.append((y4, y16))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    if S > 1:
        assert int(ws[:16384].count_nonzero()) == 0


@pytest.mark.parametrize("forced", ["1,2", "3,4", "6,2", "4,1", "6,1"])
@pytest.mark.parametrize("M", [5, 16, 29])
def test_stream_kernels_with_k_slices(env, plan, M, forced):
    """Streaming (M <= 32) kernels with every tile count, alone and with K-slices
    that meet in the workspace; 11 groups do not divide by the slice count and the
    last tile block is ragged."""
    torch, B = env
    N, K = 400, 1408
    plan("QSPEC_STREAM_W4A4", forced)
    plan("QSPEC_STREAM_W4A16", forced)
    codes, scales, x = synth.generic_case(700 + M, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    qa, sa, q_ref, s_ref = _check_quant(torch, B, x)
    ws = B.alloc_workspace(B.workspace_bytes(M, N, K))
    ref4 = orc.gemm_w4a4(q_ref, s_ref, codes, scales)
    ref16 = orc.gemm_w4a16(x, codes, scales)
    xd = dev(torch, x)
    outs = []
    for _ in range(2):
        y4 = B.gemm_w4a4(blob, qa, sa, N, workspace=ws)
        y16 = B.gemm_w4a16(blob, xd, N, workspace=ws)
        torch.cuda.synchronize()
        assert rel_err(y4.cpu().numpy(), ref4) <= TOL
        assert rel_err(y16.cpu().numpy(), ref16) <= TOL
        outs.append((y4, y16))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert int(ws[:16384].count_nonzero()) == 0


@pytest.mark.parametrize("forced", [None, "2,1,2", "4,1,2", "6,1,2", "1,1,2", "2,1,4"])
@pytest.mark.parametrize("M", [17, 29, 32, 33, 47, 64, 65, 100, 128])
def test_stream_kernels_with_token_row_blocks(env, plan, M, forced):
    """Token rows dealt to two or more workgroups that own the same weight tiles:
    forced plans with every tile count, and the library's own choice (None) on a
    narrow layer, where it picks row blocks up to 128 tokens.  Ragged M: the last
    block holds fewer rows than the others, or none at all.  (A forced plan that has
    no instance for this M falls back to the library's choice.)"""
    torch, B = env
    N, K = 400, 1408
    if forced is not None:
        plan("QSPEC_STREAM_W4A4", forced)
        plan("QSPEC_STREAM_W4A16", forced)
    codes, scales, x = synth.generic_case(900 + M, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    qa, sa, q_ref, s_ref = _check_quant(torch, B, x)
    ws = B.alloc_workspace(B.workspace_bytes(M, N, K))
    guard = 321.0
    buf4 = torch.full((M * N + 256,), guard, dtype=torch.float16, device="cuda")
    buf16 = torch.full((M * N + 256,), guard, dtype=torch.float16, device="cuda")
    y4 = B.gemm_w4a4(blob, qa, sa, N, y=buf4[128:128 + M * N].view(M, N), workspace=ws)
    torch.cuda.synchronize()
    assert rel_err(y4.cpu().numpy(), orc.gemm_w4a4(q_ref, s_ref, codes, scales)) <= TOL
    assert (buf4[:128] == guard).all() and (buf4[-128:] == guard).all()
    y16 = B.gemm_w4a16(blob, dev(torch, x), N, y=buf16[128:128 + M * N].view(M, N), workspace=ws)
    torch.cuda.synchronize()
    assert rel_err(y16.cpu().numpy(), orc.gemm_w4a16(x, codes, scales)) <= TOL
    assert (buf16[:128] == guard).all() and (buf16[-128:] == guard).all()
    if forced is None:      # one round of workgroups covers this small layer: the streaming kernel takes it in both modes
        assert B.describe_kernel(True, M, N, K).startswith("gemm_stream_kernel")
        assert B.describe_kernel(False, M, N, K).startswith("gemm_stream_kernel")


def test_tile_kernel_exact_cases(env, plan):
    """Exactly representable products through the tiled kernels with K-slices:
    any summation order must give the oracle's bits."""
    torch, B = env
    M, N, K = 100, 96, 512
    plan("QSPEC_TILE_W4A4", "1,2")
    plan("QSPEC_TILE_W4A16", "1,2")
    rng = np.random.default_rng(8)
    x = rng.integers(-2, 3, size=(M, K)).astype(np.float16)
    qw = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    sw = np.tile(np.array([[2.0 ** -6, 2.0 ** -5, 2.0 ** -7, 2.0 ** -6]], np.float16), (N, 1))
    blob = B.pack_weights(dev(torch, qw), dev(torch, sw))
    y = B.gemm_w4a16(blob, dev(torch, x), N).cpu().numpy()
    assert np.array_equal(y, orc.gemm_w4a16(x, qw, sw))
    q = rng.integers(-2, 3, size=(M, K), dtype=np.int8)
    qs = rng.integers(-2, 3, size=(N, K), dtype=np.int8)
    ones_w = np.ones((N, K // 128), np.float16)
    ones_a = np.ones((M, K // 128), np.float32)
    blob = B.pack_weights(dev(torch, qs), dev(torch, ones_w))
    y = B.gemm_w4a4(blob, dev(torch, lay.act_bytes(q)), dev(torch, ones_a), N).cpu().numpy()
    assert np.array_equal(y.astype(np.int64), q.astype(np.int64) @ qs.astype(np.int64).T)


# ------------------------------------------------------------------ the five configurations
def _rel_err_all_columns(y, ref_columns, N, chunk=2048):
    """max|y - ref| / max|ref| over ALL N columns; the oracle is evaluated in column chunks
    (ref_columns(cols) -> fp16 [M, len(cols)]) so that its float64 temporaries stay small."""
    num, den = 0.0, 0.0
    for c0 in range(0, N, chunk):
        cols = np.arange(c0, min(N, c0 + chunk))
        ref = ref_columns(cols).astype(np.float64)
        num = max(num, float(np.max(np.abs(y[:, cols].astype(np.float64) - ref))))
        den = max(den, float(np.max(np.abs(ref))))
    return num / max(den, 1e-30)


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_benchmark_configuration(env, config):
    """Full-size layers of each configuration, in the launch configuration the benchmark
    times (the library's own plan).  The packed blob is compared byte for byte, activation
    codes and scales bit for bit, partials on a 64-column window per layer, and the fp16
    outputs of both modes on EVERY element against the float64 oracle."""
    torch, B = env
    cfg = synth.CONFIGS[config]
    for li, layer in enumerate(cfg.layers):
        N, K = layer.N, layer.K
        print(f"config {config} layer {layer.name} K={K} N={N}", flush=True)
        codes = synth.weight_codes(config, li, N, K)
        scales = synth.weight_scales(config, li, N, K)
        blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
        assert np.array_equal(blob.cpu().numpy(), lay.weight_blob(codes, scales))

        # draft: quant_act + W4A4 at M = batch
        xd = synth.activations(config, li, cfg.draft_M, K, verify=False)
        qa, sa, q_ref, s_ref = _check_quant(torch, B, xd)
        n0 = (N // 2) // 16 * 16
        P = B.gemm_w4a4_partials(blob, qa, N, n0, 64).cpu().numpy()
        assert np.array_equal(P, orc.partials(q_ref, codes[n0:n0 + 64]))
        y4 = B.gemm_w4a4(blob, qa, sa, N).cpu().numpy()
        e4 = _rel_err_all_columns(y4, lambda cols: orc.gemm_w4a4_columns(q_ref, s_ref, codes, scales, cols), N)
        if B.w4a4_takes_wide(cfg.draft_M, N, K):
            # the widened activation format (what the benchmark's step feeds this layer): codes bit
            # for bit against the oracle's layout, outputs against the oracle like the packed path
            qa8, sa8 = B.quant_act_wide(dev(torch, xd))
            assert np.array_equal(qa8.cpu().numpy(), lay.act_wide_bytes(q_ref))
            assert np.array_equal(sa8.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
            y4w = B.gemm_w4a4_wide(blob, qa8, sa8, N).cpu().numpy()
            e4w = _rel_err_all_columns(y4w, lambda cols: orc.gemm_w4a4_columns(q_ref, s_ref, codes, scales, cols), N)
            print(f"   widened activations: rel err {e4w:.2e}", flush=True)
            assert e4w <= TOL

        # verify: W4A16 at M = batch * (gamma + 1)
        xv = synth.activations(config, li, cfg.verify_M, K, verify=True)
        y16 = B.gemm_w4a16(blob, dev(torch, xv), N).cpu().numpy()
        e16 = _rel_err_all_columns(y16, lambda cols: orc.gemm_w4a16_columns(xv, codes, scales, cols), N)
        print(f"   rel err w4a4 {e4:.2e}  w4a16 {e16:.2e}  ({B.describe_kernel(True, cfg.draft_M, N, K)}, "
              f"{B.describe_kernel(False, cfg.verify_M, N, K)})", flush=True)
        assert np.isfinite(y4).all() and np.isfinite(y16).all()
        assert e4 <= TOL and e16 <= TOL

        # both modes at the other mode's M as well (same-shape comparison rows of the benchmark)
        y16d = B.gemm_w4a16(blob, dev(torch, xd), N).cpu().numpy()
        e16d = _rel_err_all_columns(y16d, lambda cols: orc.gemm_w4a16_columns(xd, codes, scales, cols), N)
        qv, sv = B.quant_act(dev(torch, xv))
        qv_ref, sv_ref = orc.quant_act(xv)
        assert np.array_equal(qv.cpu().numpy(), lay.act_bytes(qv_ref))
        y4v = B.gemm_w4a4(blob, qv, sv, N).cpu().numpy()
        e4v = _rel_err_all_columns(y4v, lambda cols: orc.gemm_w4a4_columns(qv_ref, sv_ref, codes, scales, cols), N)
        if B.w4a4_takes_wide(cfg.verify_M, N, K):
            qv8, sv8 = B.quant_act_wide(dev(torch, xv))
            assert np.array_equal(qv8.cpu().numpy(), lay.act_wide_bytes(qv_ref))
            y4vw = B.gemm_w4a4_wide(blob, qv8, sv8, N).cpu().numpy()
            e4vw = _rel_err_all_columns(y4vw, lambda cols: orc.gemm_w4a4_columns(qv_ref, sv_ref, codes, scales, cols), N)
            assert e4vw <= TOL
        print(f"   at the other mode's M: w4a16 {e16d:.2e}  w4a4 {e4v:.2e}", flush=True)
        assert e16d <= TOL and e4v <= TOL
        del blob, codes


# ------------------------------------------------------------------ robustness
def test_outputs_stay_inside_their_buffers_and_are_deterministic(env):
    torch, B = env
    M, N, K = 19, 176, 640
    codes, scales, x = synth.generic_case(77, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    xd = dev(torch, x)
    pad = 256
    canary = 0x5A

    def guarded(nbytes):
        buf = torch.full((nbytes + 2 * pad,), canary, dtype=torch.uint8, device="cuda")
        return buf, buf[pad:pad + nbytes]

    qbuf, qv = guarded(M * K // 2)
    sbuf, sv = guarded(M * (K // 128) * 4)
    ybuf, yv = guarded(M * N * 2)
    zbuf, zv = guarded(M * N * 2)
    qa = qv.view(M, K // 2)
    sa = sv.view(torch.float32).view(M, K // 128)
    y4 = yv.view(torch.float16).view(M, N)
    y16 = zv.view(torch.float16).view(M, N)
    B.quant_act(xd, qa, sa)
    B.gemm_w4a4(blob, qa, sa, N, y=y4)
    B.gemm_w4a16(blob, xd, N, y=y16)
    torch.cuda.synchronize()
    for buf in (qbuf, sbuf, ybuf, zbuf):
        b = buf.cpu().numpy()
        assert (b[:pad] == canary).all() and (b[-pad:] == canary).all()
    first = (y4.clone(), y16.clone(), qa.clone())
    B.quant_act(xd, qa, sa)
    B.gemm_w4a4(blob, qa, sa, N, y=y4)
    B.gemm_w4a16(blob, xd, N, y=y16)
    torch.cuda.synchronize()
    assert torch.equal(first[0], y4) and torch.equal(first[1], y16) and torch.equal(first[2], qa)


def test_calls_on_a_side_stream(env):
    torch, B = env
    M, N, K = 8, 256, 1024
    codes, scales, x = synth.generic_case(78, M, N, K)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
        y = B.gemm_w4a16(blob, dev(torch, x), N)
    s.synchronize()
    assert rel_err(y.cpu().numpy(), orc.gemm_w4a16(x, codes, scales)) <= TOL


def test_missing_workspace_is_refused(env, plan):
    """A plan with K-slices needs the workspace: none, or a short one, is an error
    and nothing is launched."""
    torch, B = env
    M, N, K = 100, 64, 1024
    plan("QSPEC_TILE_W4A16", "2,2")
    codes, scales, x = synth.generic_case(80, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    xd = dev(torch, x)
    need = B.workspace_bytes(M, N, K)
    assert need > 16384
    y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    L = B.lib()
    assert L.qspec_gemm_w4a16(blob.data_ptr(), xd.data_ptr(), M, N, K, 128, y.data_ptr(), None, 0, None) == B.ERR_WORKSPACE
    short = torch.zeros(need - 16, dtype=torch.uint8, device="cuda")
    assert L.qspec_gemm_w4a16(blob.data_ptr(), xd.data_ptr(), M, N, K, 128, y.data_ptr(), short.data_ptr(),
                              short.numel(), None) == B.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())


def test_bad_arguments_are_refused_on_device(env):
    torch, B = env
    M, N, K = 4, 64, 256
    codes, scales, x = synth.generic_case(79, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    xd = dev(torch, x)
    L = B.lib()
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    assert L.qspec_gemm_w4a16(blob.data_ptr(), xd.data_ptr() + 2, M, N, K, 128, y.data_ptr(), None, 0, None) == B.ERR_ALIGN
    assert L.qspec_gemm_w4a16(blob.data_ptr(), xd.data_ptr(), M, N + 8, K, 128, y.data_ptr(), None, 0, None) == B.ERR_SHAPE
    with pytest.raises(B.QSpecError):
        B.quant_act(xd[:, :200].contiguous())


# ------------------------------------------------------------------ many shapes
def test_random_shapes_take_every_plan_and_match(env):
    """150 seeded shapes across the planner's regimes (streaming kernels with 1..6 tiles,
    K-slices, token-row blocks, the wide one-round plans, tiled kernels of every size
    class): both modes against the oracle, and the set of kernels that ran is reported."""
    torch, B = env
    rng = np.random.default_rng(2024)
    seen = {}
    worst = (0.0, None)
    for case in range(150):
        regime = case % 5
        if regime == 0:      # decoding batch, wide and narrow layers
            M, N, K = int(rng.integers(1, 33)), 16 * int(rng.integers(1, 700)), 128 * int(rng.integers(1, 24))
        elif regime == 1:    # mid batch
            M, N, K = int(rng.integers(33, 130)), 16 * int(rng.integers(1, 400)), 128 * int(rng.integers(1, 16))
        elif regime == 2:    # many tokens
            M, N, K = int(rng.integers(130, 700)), 16 * int(rng.integers(1, 80)), 128 * int(rng.integers(1, 10))
        elif regime == 3:    # long K, few columns (K-slices)
            M, N, K = int(rng.integers(1, 140)), 16 * int(rng.integers(1, 24)), 128 * int(rng.integers(24, 90))
        else:                # tiny
            M, N, K = int(rng.integers(1, 20)), 16 * int(rng.integers(1, 6)), 128 * int(rng.integers(1, 4))
        while M * N * K > 3e8:
            N = max(16, N // 2 // 16 * 16)
        codes, scales, x = synth.generic_case(9000 + case, M, N, K)
        blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
        xd = dev(torch, x)
        qa, sa = B.quant_act(xd)
        y4 = B.gemm_w4a4(blob, qa, sa, N).cpu().numpy()
        y16 = B.gemm_w4a16(blob, xd, N).cpu().numpy()
        q_ref, s_ref = orc.quant_act(x)
        e4 = rel_err(y4, orc.gemm_w4a4(q_ref, s_ref, codes, scales))
        e16 = rel_err(y16, orc.gemm_w4a16(x, codes, scales))
        for w4a4 in (True, False):
            k = B.describe_kernel(w4a4, M, N, K)
            seen[k] = seen.get(k, 0) + 1
        if max(e4, e16) > worst[0]:
            worst = (max(e4, e16), (M, N, K))
        assert e4 <= TOL and e16 <= TOL, (case, M, N, K, e4, e16, B.describe_kernel(True, M, N, K), B.describe_kernel(False, M, N, K))
    print("worst", worst, flush=True)
    for k in sorted(seen):
        print(f"  {seen[k]:4d}  {k}", flush=True)
    assert len(seen) >= 12            # the sample reaches a broad set of instances
