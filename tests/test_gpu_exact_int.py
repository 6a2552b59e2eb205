"""Integer stage of the PRODUCTION draft-mode kernels, bit for bit.

The debug entry that returns int32 partials runs a kernel of its own; what the hot
kernels (every streaming instance, every tiled workgroup shape, with and without
K-slices) do between the matrix instruction and the fp16 store is checked here without
any summation order: every token row has exactly ONE live group (all other activation
codes are zero, so their partial sums are exactly 0), activation and weight scales are
powers of two, and so  y[m, n] = fp16_rne(P[m, n, g*] * sa * sw)  must match the oracle
bit for bit.  Codes span the full range: weights -8 .. 7 with rows of all -8 and all 7,
activations -7 .. 7 with rows of all 7 and all -7, so |P| reaches 128 * 56 = 7168, the
extreme of the accumulator-seed trick of the streaming kernel."""
import numpy as np
import pytest

from oracle import device_layout as lay
from oracle import qspec_oracle as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2410_11305_amd import binding as B
    assert torch.cuda.is_available()
    B.lib()
    return torch, B


def _one_live_group_case(seed, M, N, G):
    rng = np.random.default_rng(seed)
    K = 128 * G
    qw = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    qw[0] = -8
    qw[1] = 7
    qw[N - 1] = -8
    qa = np.zeros((M, K), np.int8)
    for m in range(M):
        g = (m * 5 + 3) % G                      # every group is live in some row once M >= G
        row = rng.integers(-7, 8, size=128, dtype=np.int8)
        if m % 7 == 0:
            row[:] = 7
        if m % 7 == 3:
            row[:] = -7
        qa[m, 128 * g:128 * g + 128] = row
    # scales of EVERY group are non-zero powers of two: a dead group must contribute exactly 0
    sa = (2.0 ** rng.integers(-3, 3, size=(M, G))).astype(np.float32)
    sw = (2.0 ** rng.integers(-9, -5, size=(N, G))).astype(np.float16)
    return qa, sa, qw, sw


def _run_and_compare(torch, B, qa, sa, qw, sw, expect_kernel):
    M, K = qa.shape
    N = qw.shape[0]
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    blob = B.pack_weights(to(qw), to(sw))
    ws = B.alloc_workspace(B.workspace_bytes(M, N, K))
    name = B.describe_kernel(True, M, N, K)
    assert name.startswith(expect_kernel), (name, expect_kernel)
    y = B.gemm_w4a4(blob, to(lay.act_bytes(qa)), to(sa), N, workspace=ws).cpu().numpy()
    ref = orc.gemm_w4a4(qa, sa, qw, sw)
    P = orc.partials(qa, qw)
    assert np.abs(P).max() == 7168                       # the extreme is in the case
    bad = np.argwhere(y.view(np.uint16) != ref.view(np.uint16))
    assert bad.size == 0, (name, len(bad), bad[:5], y[tuple(bad[0])], ref[tuple(bad[0])])
    return name


STREAM_INSTANCES = [(tm, nt) for tm in (1, 2, 4, 8) for nt in (1, 2, 3, 4, 6) if nt * tm <= 16]


@pytest.mark.parametrize("S", [1, 2])
@pytest.mark.parametrize("tm,nt", STREAM_INSTANCES)
def test_stream_instances_integer_stage_bit_exact(env, plan, tm, nt, S):
    torch, B = env
    M = 16 * tm - 3                                      # ragged last token tile
    G = 17                                               # wave 0 takes three groups, the others two
    N = 16 * (3 * nt + 1)                                # ragged last tile block
    plan("QSPEC_STREAM_MAX_W4A4", "128")                 # lets the streaming kernel take up to 128 tokens
    plan("QSPEC_STREAM_W4A4", f"{nt},{S}")
    qa, sa, qw, sw = _one_live_group_case(100 * tm + nt, M, N, G)
    _run_and_compare(torch, B, qa, sa, qw, sw, f"gemm_stream_kernel<true, {tm}, {nt}>")


@pytest.mark.parametrize("S", [1, 2])
@pytest.mark.parametrize("shape", range(4))
def test_tile_shapes_integer_stage_bit_exact(env, plan, shape, S):
    torch, B = env
    M, N, G = 150, 304, 9                                # ragged M and N, three rounds of the 3-deep ring
    plan("QSPEC_TILE_W4A4", f"{shape},{S}")
    qa, sa, qw, sw = _one_live_group_case(500 + shape, M, N, G)
    _run_and_compare(torch, B, qa, sa, qw, sw, "gemm_tile4w_kernel")


def test_library_chosen_kernels_integer_stage_bit_exact(env):
    """The same check without any forced plan, on shapes that reach the streaming kernel,
    its token-row blocks and the tiled kernel by the library's own choice."""
    torch, B = env
    seen = set()
    for seed, (M, N, G) in enumerate([(8, 512, 9), (29, 4096, 8), (64, 1024, 12), (100, 400, 11),
                                      (128, 12288, 8), (260, 640, 10), (512, 1024, 16)]):
        qa, sa, qw, sw = _one_live_group_case(900 + seed, M, N, G)
        seen.add(_run_and_compare(torch, B, qa, sa, qw, sw, "gemm_"))
    assert any(k.startswith("gemm_tile4w_kernel") for k in seen) and any(k.startswith("gemm_stream_kernel") for k in seen)
