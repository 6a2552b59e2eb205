"""The entry point that allocates nothing (qspec_gemm_w4a16_noalloc), through the C ABI:
its output against qspec_gemm_w4a16 with a caller-provided workspace, on two calls in a
row that share the library's built-in scratch, the second on a smaller problem.  Both
shapes are planned with K-slices, so the scratch (arrival counters and partial sums) is
really used; the kernels are the same and deterministic, so the outputs must be equal
bit for bit, and both are held to the oracle's tolerance as well."""
import numpy as np
import pytest

from oracle import qspec_oracle as orc
from paper_2410_11305_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _case(torch, B, seed, M, N, K):
    codes, scales, x = synth.generic_case(seed, M, N, K)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    blob = B.pack_weights(to(codes), to(scales))
    return codes, scales, x, blob, to(x)


def test_noalloc_entry_point_matches_the_workspace_entry_point():
    import torch
    from paper_2410_11305_amd import binding as B
    assert torch.cuda.is_available()
    L = B.lib()
    shapes = [(200, 1024, 4096), (140, 512, 2048)]        # the second call is the smaller one
    for seed, (M, N, K) in enumerate(shapes):
        need = B.workspace_bytes(M, N, K)
        assert 16384 < need <= B.NOALLOC_SCRATCH_BYTES, (M, N, K, need)     # K-slices: the scratch is used
        codes, scales, x, blob, xd = _case(torch, B, 4200 + seed, M, N, K)
        ws = B.alloc_workspace(need)
        y_ws = torch.empty((M, N), dtype=torch.float16, device="cuda")
        y_na = torch.full((M, N), 123.0, dtype=torch.float16, device="cuda")
        st = L.qspec_gemm_w4a16(blob.data_ptr(), xd.data_ptr(), M, N, K, 128, y_ws.data_ptr(),
                                ws.data_ptr(), ws.numel(), None)
        assert st == B.OK
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        st = L.qspec_gemm_w4a16_noalloc(blob.data_ptr(), xd.data_ptr(), M, N, K, 128, y_na.data_ptr(), None)
        assert st == B.OK
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(y_ws, y_na)
        ref = orc.gemm_w4a16(x, codes, scales).astype(np.float64)
        err = np.max(np.abs(y_na.cpu().numpy().astype(np.float64) - ref)) / np.max(np.abs(ref))
        assert err <= TOL, err


def test_noalloc_entry_point_refuses_what_its_scratch_cannot_hold():
    import torch
    from paper_2410_11305_amd import binding as B
    L = B.lib()
    # a shape without K-slices needs no scratch and is served; bad arguments are refused
    M, N, K = 8, 256, 1024
    codes, scales, x, blob, xd = _case(torch, B, 4300, M, N, K)
    y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    assert L.qspec_gemm_w4a16_noalloc(blob.data_ptr(), xd.data_ptr(), M, N, K, 128, y.data_ptr(), None) == B.OK
    torch.cuda.synchronize()
    assert torch.equal(y, B.gemm_w4a16(blob, xd, N))
    assert L.qspec_gemm_w4a16_noalloc(None, xd.data_ptr(), M, N, K, 128, y.data_ptr(), None) == B.ERR_NULL
    assert L.qspec_gemm_w4a16_noalloc(blob.data_ptr(), xd.data_ptr() + 2, M, N, K, 128, y.data_ptr(), None) == B.ERR_ALIGN
    assert L.qspec_gemm_w4a16_noalloc(blob.data_ptr(), xd.data_ptr(), M, N + 8, K, 128, y.data_ptr(), None) == B.ERR_SHAPE
