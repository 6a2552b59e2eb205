"""Sizes at the edge of what the entry points accept: a packed weight tensor just under
the 2 GiB that the kernels' 32-bit byte offsets reach, the largest input dimension that
goes with it, and a token count far beyond any decoding batch.  The weights are drawn on
the device (seeded); the oracle sees the sampled rows only."""
import numpy as np
import pytest

from oracle import qspec_oracle as orc

pytestmark = pytest.mark.gpu

TOL = 2e-3


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2410_11305_amd import binding as B
    assert torch.cuda.is_available()
    B.lib()
    return torch, B


def rel_err(y, ref):
    return float(np.max(np.abs(y.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


def test_weight_tensor_just_under_two_gib(env):
    torch, B = env
    N, K = 32800, 130944                      # N*K/2 = 2 147 481 600 bytes of codes (limit: 2^31 - 2)
    assert N * K // 2 < 2 ** 31 - 1 <= (N + 16) * K // 2
    G = K // 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    codes = torch.randint(-8, 8, (N, K), dtype=torch.int8, device="cuda", generator=gen)
    scales = (torch.rand((N, G), device="cuda", generator=gen) * 0.008 + 0.002).half()
    blob = B.pack_weights(codes, scales)
    assert blob.numel() == B.packed_weight_bytes(N, K) == N * K // 2 + N * G * 2
    cols = np.unique(np.concatenate([np.arange(16), np.arange(N - 16, N), [N // 2, N // 2 + 17, 12345, 30001, 32767, 32768]]))
    c_h = codes[torch.from_numpy(cols).cuda()].cpu().numpy()
    s_h = scales[torch.from_numpy(cols).cuda()].cpu().numpy()
    # the round trip of the sampled rows (first tile, last tile, middle)
    back_c, back_s = B.unpack_weights(blob, N, K)
    assert torch.equal(back_c[-16:], codes[-16:]) and torch.equal(back_c[:16], codes[:16])
    assert torch.equal(back_s, scales)
    del back_c, back_s, codes
    rng = np.random.default_rng(78)
    for M in (8, 96):                          # the streaming and the tiled kernels
        x = rng.standard_normal((M, K)).astype(np.float16)
        x[:, rng.choice(K, K // 100, replace=False)] *= 20
        xd = torch.from_numpy(x).cuda()
        qa, sa = B.quant_act(xd)
        q_ref, s_ref = orc.quant_act(x)
        assert np.array_equal(sa.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
        y4 = B.gemm_w4a4(blob, qa, sa, N)
        y16 = B.gemm_w4a16(blob, xd, N)
        torch.cuda.synchronize()
        print(M, B.describe_kernel(True, M, N, K), B.describe_kernel(False, M, N, K), flush=True)
        y4, y16 = y4.cpu().numpy(), y16.cpu().numpy()
        assert np.isfinite(y4).all() and np.isfinite(y16).all()
        e4 = rel_err(y4[:, cols], orc.gemm_w4a4(q_ref, s_ref, c_h, s_h))
        e16 = rel_err(y16[:, cols], orc.gemm_w4a16(x, c_h, s_h))
        print(f"   rel err w4a4 {e4:.2e}  w4a16 {e16:.2e}", flush=True)
        assert e4 <= TOL and e16 <= TOL


def test_one_row_too_many_is_refused(env):
    torch, B = env
    a = torch.zeros(64, dtype=torch.uint8, device="cuda")
    assert B.packed_weight_bytes(32800 + 16, 130944) == 0
    with pytest.raises(B.QSpecError):
        B.gemm_w4a16(a, torch.zeros((1, 130944), dtype=torch.float16, device="cuda"), 32800 + 16,
                     y=torch.zeros((1, 32800 + 16), dtype=torch.float16, device="cuda"))
    torch.cuda.synchronize()


def test_twenty_thousand_tokens(env):
    torch, B = env
    M, N, K = 20001, 48, 1024                 # 157 token blocks of 128, the last with one row
    rng = np.random.default_rng(79)
    codes = rng.integers(-8, 8, (N, K), dtype=np.int8)
    scales = rng.uniform(0.002, 0.01, (N, K // 128)).astype(np.float16)
    x = rng.standard_normal((M, K)).astype(np.float16)
    blob = B.pack_weights(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda())
    xd = torch.from_numpy(x).cuda()
    qa, sa = B.quant_act(xd)
    q_ref, s_ref = orc.quant_act(x)
    assert np.array_equal(sa.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    y4 = B.gemm_w4a4(blob, qa, sa, N).cpu().numpy()
    y16 = B.gemm_w4a16(blob, xd, N).cpu().numpy()
    assert rel_err(y4, orc.gemm_w4a4(q_ref, s_ref, codes, scales)) <= TOL
    assert rel_err(y16, orc.gemm_w4a16(x, codes, scales)) <= TOL
