"""The draft-pass MLP of a decoder block as one persistent launch (qspec_mlp_draft) against
the chain of oracles, stage by stage on identical inputs (paper Sec. 3.1, draft phase):
    W4A4 gate/up  ->  SiLU(gate) * up + quantiser  ->  W4A4 down
The fp16 gate/up tensor is held to the GEMM tolerance; the codes and scales of the
quantised intermediate must equal, bit for bit, the oracle's quantiser applied to the
oracle's SiLU * up of the DEVICE's gate/up tensor; the final output is held to the GEMM
tolerance against the oracle's product of those codes.  The persistent launch must also
agree bit for bit with the three separate calls it replaces."""
import numpy as np
import pytest

from oracle import device_layout as lay
from oracle import producers_oracle as prod
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


def rel(y, ref):
    return float(np.max(np.abs(y.astype(np.float64) - ref.astype(np.float64))) / max(np.max(np.abs(ref.astype(np.float64))), 1e-30))


def _case(torch, B, seed, M, H, I):
    rng = np.random.default_rng(seed)
    x, w_norm, _ = synth.producer_case(seed, M, H, 128)
    c_gu = rng.integers(-8, 8, (2 * I, H), dtype=np.int8)
    s_gu = rng.uniform(0.002, 0.01, (2 * I, H // 128)).astype(np.float16)
    c_dn = rng.integers(-8, 8, (H, I), dtype=np.int8)
    s_dn = rng.uniform(0.002, 0.01, (H, I // 128)).astype(np.float16)
    blob_gu = B.pack_weights(dev(torch, c_gu), dev(torch, s_gu))
    blob_dn = B.pack_weights(dev(torch, c_dn), dev(torch, s_dn))
    qa1, sa1, _ = B.rmsnorm_quant(dev(torch, x), dev(torch, w_norm), synth.RMS_EPS)
    return (c_gu, s_gu, c_dn, s_dn), blob_gu, blob_dn, qa1, sa1


@pytest.mark.parametrize("M,H,I", [(8, 512, 1024), (1, 128, 128), (29, 1024, 2816), (32, 1152, 3072),
                                   (8, 4096, 11008), (32, 4096, 11008)])
def test_persistent_mlp_matches_the_oracle_chain_and_the_separate_calls(env, M, H, I):
    torch, B = env
    (c_gu, s_gu, c_dn, s_dn), blob_gu, blob_dn, qa1, sa1 = _case(torch, B, 800 + M + H, M, H, I)
    ws = B.alloc_workspace(B.mlp_draft_workspace_bytes(M, H, I))
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    outs = []
    for _ in range(2):                                     # the second call finds the counters as the first left them
        gu, qa2, sa2, y = B.mlp_draft(blob_gu, blob_dn, qa1, sa1, H, I, ws, status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        outs.append((gu.clone(), qa2.clone(), sa2.clone(), y.clone()))
    assert int(ws.count_nonzero()) == 0
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    gu, qa2, sa2, y = outs[0]
    # against the oracles, stage by stage
    q1 = lay.decode_act_bytes(qa1.cpu().numpy())
    s1 = sa1.cpu().numpy()
    gu_h = gu.cpu().numpy()
    assert rel(gu_h, orc.gemm_w4a4(q1, s1, c_gu, s_gu)) <= TOL
    q2, s2 = orc.quant_act(prod.silu_mul_f16(gu_h))
    assert np.array_equal(qa2.cpu().numpy(), lay.act_bytes(q2))
    assert np.array_equal(sa2.cpu().numpy().view(np.uint32), s2.view(np.uint32))
    assert rel(y.cpu().numpy(), orc.gemm_w4a4(q2, s2, c_dn, s_dn)) <= TOL
    # against the three launches it replaces (same arithmetic per output element up to the
    # order in which the eight wavefronts' sums are added: hold it to the tolerance, and the
    # integer stage to equality given the same gate/up tensor)
    gu3 = B.gemm_w4a4(blob_gu, qa1, sa1, 2 * I)
    assert rel(gu_h, gu3.cpu().numpy()) <= TOL
    qa3, sa3, _ = B.silu_mul_quant(gu)
    assert torch.equal(qa3, qa2) and torch.equal(sa3, sa2)
    y3 = B.gemm_w4a4(blob_dn, qa2, sa2, H)
    assert rel(y.cpu().numpy(), y3.cpu().numpy()) <= TOL


def test_persistent_mlp_refuses_what_it_cannot_hold(env):
    torch, B = env
    L = B.lib()
    M, H, I = 8, 512, 1024
    _, blob_gu, blob_dn, qa1, sa1 = _case(torch, B, 900, M, H, I)
    ws = B.alloc_workspace(B.mlp_draft_workspace_bytes(M, H, I))
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    gu = torch.empty((M, 2 * I), dtype=torch.float16, device="cuda")
    qa2 = torch.empty((M, I // 2), dtype=torch.uint8, device="cuda")
    sa2 = torch.empty((M, I // 128), dtype=torch.float32, device="cuda")
    y = torch.empty((M, H), dtype=torch.float16, device="cuda")
    args = lambda m, h, i, wsb: (blob_gu.data_ptr(), blob_dn.data_ptr(), qa1.data_ptr(), sa1.data_ptr(), m, h, i, 128,
                                 gu.data_ptr(), qa2.data_ptr(), sa2.data_ptr(), y.data_ptr(), ws.data_ptr(), wsb,
                                 status.data_ptr(), None)
    assert L.qspec_mlp_draft(*args(33, H, I, ws.numel())) == B.ERR_UNSUPPORTED          # more than 32 tokens
    assert L.qspec_mlp_draft(*args(M, H, I + 64, ws.numel())) == B.ERR_SHAPE
    assert L.qspec_mlp_draft(*args(M, H, I, 64)) == B.ERR_WORKSPACE
    assert L.qspec_mlp_draft(*args(8, 8192, 28672, ws.numel())) == B.ERR_UNSUPPORTED    # 70B-shaped: does not fit LDS


def test_persistent_mlp_gives_up_cleanly_when_the_wait_is_cut_short(env, plan):
    """The wait between the stages is bounded.  With a limit of one poll, workgroups that
    arrive before the quantised activations are complete give up: they raise the status
    word and every workgroup exits (nothing hangs).  Whether any does is a matter of timing,
    so: either the status word is raised, or the result is the regular one.  Afterwards the
    workspace is cleared and a regular call works."""
    torch, B = env
    M, H, I = 8, 4096, 11008
    (c_gu, s_gu, c_dn, s_dn), blob_gu, blob_dn, qa1, sa1 = _case(torch, B, 950, M, H, I)
    ws = B.alloc_workspace(B.mlp_draft_workspace_bytes(M, H, I))
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    plan("QSPEC_MLP_SPIN", "1")
    gu, qa2, sa2, y = B.mlp_draft(blob_gu, blob_dn, qa1, sa1, H, I, ws, status)
    torch.cuda.synchronize()
    gave_up = int(status.item()) == 1
    plan("QSPEC_MLP_SPIN", None)
    ws.zero_()
    status.zero_()
    gu2, qa22, sa22, y2 = B.mlp_draft(blob_gu, blob_dn, qa1, sa1, H, I, ws, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and int(ws.count_nonzero()) == 0
    q2, s2 = orc.quant_act(prod.silu_mul_f16(gu2.cpu().numpy()))
    assert np.array_equal(qa22.cpu().numpy(), lay.act_bytes(q2))
    assert rel(y2.cpu().numpy(), orc.gemm_w4a4(q2, s2, c_dn, s_dn)) <= TOL
    if not gave_up:
        assert torch.equal(y, y2)
