"""The hot path captured into a HIP graph and replayed, as the benchmark runs it.

A graph holds the launches of one draft pass and one verify pass over a layer whose plans cut K
into slices (arrival counters in the workspace must be left zero by every replay), the widened
activation format, and the entry point that brings its own scratch.  The graph is replayed
several times with fresh activations copied into its buffers, eager calls and synchronisations
between the replays; every replay must give exactly what the eager calls give on the same data
(the kernels are deterministic), and the eager result is held to the oracle once."""
import numpy as np
import pytest

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


@pytest.mark.parametrize("M,N,K,forced", [(150, 304, 896, "3"), (8, 512, 1024, None), (130, 2048, 4096, None)])
def test_graph_replays_match_eager(env, plan, M, N, K, forced):
    torch, B = env
    if forced:
        plan("QSPEC_TILE_W4A4", f"1,{forced}")          # K-slices in both modes
        plan("QSPEC_TILE_W4A16", f"0,{forced}")
    codes, scales, x0 = synth.generic_case(1234 + M, M, N, K)
    blob = B.pack_weights(dev(torch, codes), dev(torch, scales))
    wide = B.w4a4_takes_wide(M, N, K)
    x = dev(torch, x0)
    qa = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    qa8 = torch.empty((M, K), dtype=torch.int8, device="cuda")
    sa = torch.empty((M, K // 128), dtype=torch.float32, device="cuda")
    y4 = torch.empty((M, N), dtype=torch.float16, device="cuda")
    y4w = torch.empty_like(y4)
    y16 = torch.empty_like(y4)
    y16n = torch.empty_like(y4)
    ws = B.alloc_workspace(max(B.workspace_bytes(M, N, K), 16))

    def step(out4, out4w, out16, out16n, w):
        B.quant_act(x, qa, sa)
        B.gemm_w4a4(blob, qa, sa, N, y=out4, workspace=w)
        if wide:
            B.quant_act_wide(x, qa8, sa)
            B.gemm_w4a4_wide(blob, qa8, sa, N, y=out4w, workspace=w)
        B.gemm_w4a16(blob, x, N, y=out16, workspace=w)
        B.gemm_w4a16_noalloc(blob, x, N, y=out16n)

    step(y4, y4w, y16, y16n, ws)                        # eager once: nothing first-time inside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g):
            step(y4, y4w, y16, y16n, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    e4, e4w, e16, e16n = (torch.empty_like(y4) for _ in range(4))
    ws_e = B.alloc_workspace(max(B.workspace_bytes(M, N, K), 16))
    rng = np.random.default_rng(5)
    for r in range(4):
        x_new = (x0.astype(np.float32) * np.float32(1.0 + 0.25 * r) + rng.standard_normal(x0.shape).astype(np.float32) * 0.1).astype(np.float16)
        x.copy_(dev(torch, x_new))
        for t in (y4, y4w, y16, y16n):
            t.fill_(float("nan"))                       # a replay must write everything again
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        step(e4, e4w, e16, e16n, ws_e)                  # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(y4, e4) and torch.equal(y16, e16) and torch.equal(y16n, e16), r
        if wide:
            assert torch.equal(y4w, e4w) and torch.equal(y4w, y4), r
        assert int(ws[:16384].count_nonzero()) == 0, r
        if r == 0 or r == 3:
            q_ref, s_ref = orc.quant_act(x_new)
            assert rel_err(y4.cpu().numpy(), orc.gemm_w4a4(q_ref, s_ref, codes, scales)) <= TOL
            assert rel_err(y16.cpu().numpy(), orc.gemm_w4a16(x_new, codes, scales)) <= TOL
