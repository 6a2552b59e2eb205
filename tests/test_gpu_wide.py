"""The widened activation format of the draft mode: qspec_quant_act_wide -> qspec_gemm_w4a4_wide.

Same quantiser, same product (paper Sec. 1, W4A4; Sec. 4.1, groups of 128); only the storage of
the activation codes differs (one int8 = 16 * code per code, in the order the tiled kernel's LDS
rows use), and the tiled kernel takes them global -> LDS directly.  Codes and scales are checked
bit for bit against the oracle's own statement of the layout, the product against the float64
oracle and, bit for bit, on the cases whose result involves no summation order."""
import ctypes

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
    B.lib()
    return torch, B


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(y, ref):
    return float(np.max(np.abs(y.astype(np.float64) - ref.astype(np.float64))) / max(np.max(np.abs(ref.astype(np.float64))), 1e-30))


@pytest.mark.parametrize("M,K", [(1, 128), (5, 256), (65, 1024), (128, 8192), (300, 4096)])
def test_quant_act_wide_bit_exact(env, M, K):
    torch, B = env
    x = synth.generic_case(4000 + M, M, 16, K)[2]
    q_ref, s_ref = orc.quant_act(x)
    qa8, sa = B.quant_act_wide(dev(torch, x))
    assert qa8.dtype == torch.int8 and tuple(qa8.shape) == (M, K)
    assert np.array_equal(qa8.cpu().numpy(), lay.act_wide_bytes(q_ref))
    assert np.array_equal(sa.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    # and the two formats of the quantiser hold the same codes
    qa, sa2 = B.quant_act(dev(torch, x))
    assert np.array_equal(lay.decode_act_wide_bytes(qa8.cpu().numpy()), lay.decode_act_bytes(qa.cpu().numpy()))
    assert torch.equal(sa, sa2)


def test_quant_act_wide_special_values(env):
    """Zero groups, ties, the largest and smallest fp16 magnitudes: as the packed quantiser."""
    torch, B = env
    x = np.zeros((4, 256), dtype=np.float16)
    x[0, :5] = [7, -3.5, 0.5, 1.5, 2.5]
    x[1, 128:] = 65504.0
    x[1, 130] = -65504.0
    x[2, :128] = 5.96e-8
    x[2, 7] = -5.96e-8
    x[3, 3] = 1.0
    q_ref, s_ref = orc.quant_act(x)
    qa8, sa = B.quant_act_wide(dev(torch, x))
    assert np.array_equal(qa8.cpu().numpy(), lay.act_wide_bytes(q_ref))
    assert np.array_equal(sa.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))


@pytest.mark.parametrize("S", [1, 3])
@pytest.mark.parametrize("shape", range(4))
def test_wide_product_every_workgroup_shape(env, plan, shape, S):
    """Every draft-mode workgroup shape, alone and in three K-slices, ragged M and N, a group
    count that the slices do not divide; twice over the same workspace."""
    torch, B = env
    M, N, K = 150, 304, 896
    plan("QSPEC_TILE_W4A4", f"{shape},{S}")
    codes, scales, x = synth.generic_case(700 + shape, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    q_ref, s_ref = orc.quant_act(x)
    qa8, sa = B.quant_act_wide(dev(torch, x))
    assert B.w4a4_takes_wide(M, N, K)
    ws = B.alloc_workspace(max(B.workspace_bytes(M, N, K), 16))
    ref = orc.gemm_w4a4(q_ref, s_ref, codes, scales)
    qa, sa_p = B.quant_act(dev(torch, x))
    y_packed = B.gemm_w4a4(blob, qa, sa_p, N, workspace=ws)
    outs = []
    for _ in range(2):
        y = B.gemm_w4a4_wide(blob, qa8, sa, N, workspace=ws)
        torch.cuda.synchronize()
        assert rel_err(y.cpu().numpy(), ref) <= TOL
        outs.append(y)
    assert torch.equal(outs[0], outs[1])
    assert torch.equal(outs[0], y_packed)             # same arithmetic in the same order: the same bits
    if S > 1:
        assert int(ws[:16384].count_nonzero()) == 0


@pytest.mark.parametrize("S", [1, 2])
@pytest.mark.parametrize("shape", range(4))
def test_wide_product_integer_stage_bit_exact(env, plan, shape, S):
    """One live group per token row, power-of-two scales, codes over the full range (|P| up to
    7168): y = fp16(P * sa * sw) without any summation order, bit for bit against the oracle.  The
    widened codes come from the oracle's layout, not from the GPU quantiser."""
    torch, B = env
    M, N, G = 150, 304, 9
    K = 128 * G
    plan("QSPEC_TILE_W4A4", f"{shape},{S}")
    rng = np.random.default_rng(800 + shape)
    qw = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    qw[0], qw[1], qw[N - 1] = -8, 7, -8
    qa = np.zeros((M, K), np.int8)
    for m in range(M):
        g = (m * 5 + 3) % G
        row = rng.integers(-7, 8, size=128, dtype=np.int8)
        if m % 7 == 0:
            row[:] = 7
        if m % 7 == 3:
            row[:] = -7
        qa[m, 128 * g:128 * g + 128] = row
    sa = (2.0 ** rng.integers(-3, 3, size=(M, G))).astype(np.float32)
    sw = (2.0 ** rng.integers(-9, -5, size=(N, G))).astype(np.float16)
    blob = B.pack_weights(dev(torch, qw), dev(torch, sw))
    ws = B.alloc_workspace(max(B.workspace_bytes(M, N, K), 16))
    y = B.gemm_w4a4_wide(blob, dev(torch, lay.act_wide_bytes(qa)), dev(torch, sa), N, workspace=ws).cpu().numpy()
    ref = orc.gemm_w4a4(qa, sa, qw, sw)
    assert np.abs(orc.partials(qa, qw)).max() == 7168
    bad = np.argwhere(y.view(np.uint16) != ref.view(np.uint16))
    assert bad.size == 0, (len(bad), bad[:5])


def test_wide_product_library_plans_and_ragged_shapes(env):
    """The library's own plans on shapes that reach each tiled instance, with ragged tails."""
    torch, B = env
    seen = set()
    for seed, (M, N, K) in enumerate([(65, 2064, 1024), (128, 12288, 1024), (200, 640, 3072), (257, 1040, 2048),
                                      (512, 4096, 2048), (130, 39680, 256), (384, 8192, 5376)]):
        if not B.w4a4_takes_wide(M, N, K):
            continue
        codes, scales, x = synth.generic_case(900 + seed, M, N, K)
        blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
        q_ref, s_ref = orc.quant_act(x)
        qa8, sa = B.quant_act_wide(dev(torch, x))
        y = B.gemm_w4a4_wide(blob, qa8, sa, N).cpu().numpy()
        ref = orc.gemm_w4a4(q_ref, s_ref, codes, scales)
        assert rel_err(y, ref) <= TOL, (M, N, K)
        seen.add(B.describe_kernel(True, M, N, K))
    assert len(seen) >= 2, seen


def test_wide_entry_points_refuse_what_they_cannot_do(env):
    torch, B = env
    L = B.lib()
    M, N, K = 8, 256, 512                            # a streaming-kernel shape: packed codes only
    assert not B.w4a4_takes_wide(M, N, K)
    assert B.w4a4_takes_wide(0, N, K) is False and B.w4a4_takes_wide(200, N, 100) is False
    codes, scales, x = synth.generic_case(990, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    qa8, sa = B.quant_act_wide(dev(torch, x))         # the quantiser itself takes any shape
    y = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = L.qspec_gemm_w4a4_wide(vp(blob), vp(qa8), vp(sa), M, N, K, 128, vp(y), None, 0, None)
    assert rc == B.ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())                     # nothing was launched
    assert L.qspec_gemm_w4a4_wide(None, vp(qa8), vp(sa), 200, N, K, 128, vp(y), None, 0, None) == B.ERR_NULL
    assert L.qspec_gemm_w4a4_wide(vp(blob), vp(qa8), vp(sa), 200, N, 100, 128, vp(y), None, 0, None) == B.ERR_SHAPE
    assert L.qspec_quant_act_wide(vp(y), 0, 128, 128, vp(qa8), vp(sa), None) == B.ERR_SHAPE
    assert L.qspec_quant_act_wide(vp(y), 1, 128, 128, None, vp(sa), None) == B.ERR_NULL
    assert L.qspec_quant_act_wide(ctypes.c_void_p(y.data_ptr() + 2), 1, 128, 128, vp(qa8), vp(sa), None) == B.ERR_ALIGN
