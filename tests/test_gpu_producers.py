"""GPU-vs-oracle parity of the producers fused with the activation quantiser
(RMSNorm, SiLU(gate) * up; the draft phase of paper Sec. 3.1 consumes their
output as 4-bit codes) through the C ABI.  The arithmetic is fixed on both
sides, so the fp16 tensor, the codes and the scales must match bit for bit."""
import numpy as np
import pytest

from oracle import device_layout as lay
from oracle import producers_oracle as prod
from oracle import qspec_oracle as orc
from oracle import rotation_oracle as rot
from paper_2410_11305_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2410_11305_amd import binding as B
    assert torch.cuda.is_available()
    B.lib()
    return torch, B


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_against(torch, qa, sa, h, h_ref):
    """The fused launch must equal the oracle's quantiser applied to the oracle's fp16 tensor."""
    q_ref, s_ref = orc.quant_act(h_ref)
    torch.cuda.synchronize()
    if h is not None:
        assert np.array_equal(h.cpu().numpy().view(np.uint16), h_ref.view(np.uint16))
    assert np.array_equal(sa.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(qa.cpu().numpy(), lay.act_bytes(q_ref))


def check_wide_against(torch, qa8, sa, h_ref):
    """The same launch asked for the widened code format: the same codes, one byte each."""
    q_ref, s_ref = orc.quant_act(h_ref)
    torch.cuda.synchronize()
    assert np.array_equal(sa.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(qa8.cpu().numpy(), lay.act_wide_bytes(q_ref))


def run_rmsnorm(env, x, w, eps, want_h=True, rotate=False):
    torch, B = env
    qa, sa, h = B.rmsnorm_quant(dev(torch, x), dev(torch, w), eps, want_h=want_h, rotate=rotate)
    h_ref = prod.rmsnorm_f16(x, w, eps)
    h_ref = rot.hadamard128_f16(h_ref) if rotate else h_ref
    check_against(torch, qa, sa, h, h_ref)
    qa8, sa8, _ = B.rmsnorm_quant(dev(torch, x), dev(torch, w), eps, rotate=rotate, wide=True)
    check_wide_against(torch, qa8, sa8, h_ref)
    return qa, sa


def run_silu(env, gu, want_h=True, rotate=False):
    torch, B = env
    qa, sa, h = B.silu_mul_quant(dev(torch, gu), want_h=want_h, rotate=rotate)
    h_ref = prod.silu_mul_f16(gu)
    h_ref = rot.hadamard128_f16(h_ref) if rotate else h_ref
    check_against(torch, qa, sa, h, h_ref)
    qa8, sa8, _ = B.silu_mul_quant(dev(torch, gu), rotate=rotate, wide=True)
    check_wide_against(torch, qa8, sa8, h_ref)
    return qa, sa


# K: less than a wavefront's worth, ragged last wavefront, the hidden sizes of the
# configurations (one pass of up to 1024 threads), two and four passes with ragged tails,
# and more than the register-resident limit (32768)
@pytest.mark.parametrize("M,K", [(1, 128), (3, 256), (5, 2048), (4, 2176), (8, 4096), (64, 5120), (128, 8192),
                                 (2, 16384), (3, 16512), (2, 28672), (2, 33024), (300, 384)])
def test_rmsnorm_quant_bit_exact(env, M, K):
    x, w, _ = synth.producer_case(300 + M + K, M, K, 128)
    run_rmsnorm(env, x, w, synth.RMS_EPS)
    run_rmsnorm(env, x, w, synth.RMS_EPS, want_h=False)
    run_rmsnorm(env, x, w, synth.RMS_EPS, rotate=True)


def test_rmsnorm_quant_special_rows(env):
    K = 512
    rng = np.random.default_rng(7)
    x = np.zeros((7, K), dtype=np.float16)
    x[1] = 3.0                                              # constant row
    x[2, 77] = -0.5                                         # one-hot
    x[3] = rng.standard_normal(K) * 6e-5                    # fp16 subnormals, eps dominates
    x[4] = rng.standard_normal(K) * 2000.0                  # large magnitudes
    x[5, :128] = rng.standard_normal(128)                   # three all-zero groups
    x[6] = rng.standard_normal(K)
    w = (1.0 + 0.25 * rng.standard_normal(K)).astype(np.float16)
    for eps in (1e-6, 1e-5, 12.0):
        run_rmsnorm(env, x, w, eps)
    run_rmsnorm(env, x[1:3], w, 0.0)                        # eps = 0 on rows that are not zero


@pytest.mark.parametrize("M,I", [(1, 128), (3, 384), (8, 11008), (64, 13824), (128, 28672), (515, 256)])
def test_silu_mul_quant_bit_exact(env, M, I):
    _, _, gu = synth.producer_case(400 + M + I, M, 128, I)
    run_silu(env, gu)
    run_silu(env, gu, want_h=False)
    run_silu(env, gu, rotate=True)


def test_silu_mul_quant_whole_gate_range(env):
    """Every finite fp16 bit pattern as a gate value (both signs), against a few up values."""
    bits = np.concatenate([np.arange(0, 0x7C00, dtype=np.uint16), np.arange(0x8000, 0xFC00, dtype=np.uint16)])
    gate = np.resize(bits.view(np.float16), (62, 1024))
    rng = np.random.default_rng(8)
    up = np.resize(np.array([1.0, -0.5, 0.001, 0.75], np.float16), (62, 1024)) * \
        rng.choice(np.array([1, 1, 0.5], np.float16), size=(62, 1024))
    gu = np.concatenate([gate, up.astype(np.float16)], axis=1)
    with np.errstate(over="ignore", invalid="ignore"):
        h_ref = prod.silu_mul_f16(gu)
    finite = np.isfinite(h_ref.astype(np.float32)).all(axis=1)      # fp16 overflow of g * u is out of contract
    run_silu(env, gu[finite])


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_producers_on_benchmark_shapes_feed_the_draft_gemm(env, config):
    """Draft-pass shapes of every configuration; the codes of the fused RMSNorm go
    through the draft-mode GEMM of the first layer and must give what the quantiser's
    own codes give (same bytes in, same kernel)."""
    torch, B = env
    x, w, gu = synth.producer_inputs(config)
    qa, sa = run_rmsnorm(env, x, w, synth.RMS_EPS)
    run_silu(env, gu)
    layer = synth.CONFIGS[config].layers[0]
    N = min(layer.N, 1024)
    codes = synth.weight_codes(config, 0, layer.N, layer.K)[:N]
    scales = synth.weight_scales(config, 0, layer.N, layer.K)[:N]
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    h = dev(torch, prod.rmsnorm_f16(x, w, synth.RMS_EPS))
    qa2, sa2 = B.quant_act(h)
    y1 = B.gemm_w4a4(blob, qa, sa, N)
    y2 = B.gemm_w4a4(blob, qa2, sa2, N)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)


def run_hadamard(env, x, want_h=True):
    torch, B = env
    qa, sa, h = B.hadamard_quant(dev(torch, x), want_h=want_h)
    check_against(torch, qa, sa, h, rot.hadamard128_f16(x))
    return qa, sa, h


@pytest.mark.parametrize("M,K", [(1, 128), (3, 256), (5, 1024), (8, 4096), (32, 11008), (128, 28672), (515, 384)])
def test_hadamard_quant_bit_exact(env, M, K):
    _, _, x = synth.generic_case(500 + M + K, M, 16, K)
    run_hadamard(env, x)
    run_hadamard(env, x, want_h=False)


def test_hadamard_quant_special_rows(env):
    K = 256
    rng = np.random.default_rng(9)
    x = np.zeros((8, K), dtype=np.float16)
    x[1, 5] = 8.0                                          # one-hot: a row of the matrix, +-1
    x[2] = 1.0                                             # constant: only entry 0 of each group survives (16)
    x[3] = rng.integers(-40, 41, K)                        # integers: every sum exact
    x[4] = rng.standard_normal(K) * 6e-5                   # subnormal neighbourhood
    x[5] = rng.standard_normal(K) * 400.0                  # sums near the top of the fp16 range / 8
    x[6, 128:] = rng.standard_normal(128)                  # first group all zero
    x[7] = rng.standard_normal(K)
    x[7, 200] = 90.0                                       # one dominant channel
    _, _, h = run_hadamard(env, x)
    h = h.cpu().numpy()
    assert sorted(set(np.abs(h[1, :128]).tolist())) == [1.0] and not h[1, 128:].any()
    assert h[2, 0] == 16 and h[2, 128] == 16 and np.count_nonzero(h[2]) == 2


def test_rotated_activations_give_the_same_product_with_rotated_weights(env):
    """x' = x H / 8 and w' = w H / 16 per group: x' w'^T = x w^T.  Checked end to end on the
    device in verify mode with weights whose rotated form is exactly representable (every
    group of a weight row is a signed row of H, so w H / 16 is 8 times a unit vector)."""
    torch, B = env
    from scipy.linalg import hadamard
    H = hadamard(128).astype(np.int64)
    rng = np.random.default_rng(10)
    N, K, M = 64, 512, 24
    G = K // 128
    pick = rng.integers(0, 128, (N, G))
    sign = rng.choice([-1, 1], (N, G))
    codes_plain = (H[pick] * sign[:, :, None]).reshape(N, K).astype(np.int8)          # entries +-1
    codes_rot = np.zeros((N, G, 128), dtype=np.int8)
    np.put_along_axis(codes_rot, pick[:, :, None], (8 * sign)[:, :, None].astype(np.int8), axis=2)
    codes_rot = codes_rot.reshape(N, K)        # (w_g H / 16): 128 / 16 = 8 at the picked position... as a code of scale 1
    scales = np.ones((N, G), dtype=np.float16)
    # the code range stops at 7: carry the factor in the scale instead (code 4, scale 2)
    codes_rot = (codes_rot // 2).astype(np.int8)
    scales_rot = np.full((N, G), 2.0, dtype=np.float16)
    x = rng.integers(-20, 21, (M, K)).astype(np.float16)
    _, _, h = B.hadamard_quant(dev(torch, x), want_h=True)
    y_plain = B.gemm_w4a16(B.pack_weights(dev(torch, codes_plain), dev(torch, scales)), dev(torch, x), N)
    y_rot = B.gemm_w4a16(B.pack_weights(dev(torch, codes_rot), dev(torch, scales_rot)), h, N)
    torch.cuda.synchronize()
    ref = x.astype(np.float64) @ codes_plain.astype(np.float64).T
    assert np.array_equal(y_plain.cpu().numpy().astype(np.float64), ref.astype(np.float16).astype(np.float64))
    assert torch.equal(y_plain, y_rot)


def test_random_shapes_all_producers(env):
    """60 seeded shapes: every fused kernel, with and without the rotation, against the oracles."""
    rng = np.random.default_rng(31)
    for case in range(60):
        M = int(rng.integers(1, 200))
        K = 128 * int(rng.integers(1, 70))
        I = 128 * int(rng.integers(1, 40))
        x, w, gu = synth.producer_case(800 + case, M, K, I)
        rotate = bool(case & 1)
        run_rmsnorm(env, x, w, [1e-6, 1e-5, 0.25][case % 3], want_h=bool(case & 2), rotate=rotate)
        run_silu(env, gu, want_h=bool(case & 2), rotate=rotate)
        if case % 4 == 0:
            run_hadamard(env, x)


def test_bad_arguments_are_refused(env):
    torch, B = env
    x = torch.zeros((2, 256), dtype=torch.float16, device="cuda")
    w = torch.ones((256,), dtype=torch.float16, device="cuda")
    with pytest.raises(B.QSpecError):
        B.rmsnorm_quant(x, w, -1.0)
    with pytest.raises(B.QSpecError):
        B.rmsnorm_quant(x, w, float("nan"))
    with pytest.raises(B.QSpecError):
        B.rmsnorm_quant(x[:, :192].contiguous(), w[:192].contiguous(), 1e-5)      # K not a multiple of 128
    with pytest.raises(B.QSpecError):
        B.silu_mul_quant(torch.zeros((2, 2 * 192), dtype=torch.float16, device="cuda"))
    with pytest.raises(B.QSpecError):
        B.hadamard_quant(torch.zeros((2, 192), dtype=torch.float16, device="cuda"))
    torch.cuda.synchronize()
