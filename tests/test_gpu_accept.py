"""GPU-vs-oracle parity of the steps after the verify pass (greedy acceptance,
KV-cache overwrite; paper Sec. 3.1) through the C ABI.  Integer and byte work:
everything must match bit for bit."""
import numpy as np
import pytest

from oracle import accept_oracle as acc
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


def run_accept(env, logits, draft):
    torch, B = env
    n, out = B.greedy_accept(dev(torch, logits), dev(torch, draft))
    torch.cuda.synchronize()
    return n.cpu().numpy(), out.cpu().numpy()


@pytest.mark.parametrize("B_,gamma,V", [(1, 1, 1), (1, 1, 8), (3, 2, 17), (4, 3, 1024), (5, 5, 4104), (2, 4, 12345),
                                        (7, 3, 32000), (2, 3, 128256), (9, 1, 65), (1, 7, 262144 + 8)])
def test_accept_matches_oracle(env, B_, gamma, V):
    logits, draft, planted = synth.accept_case(100 + V % 97, B_, gamma, V, p_accept=0.7)
    a_ref, out_ref = acc.greedy_accept(logits, draft)
    a, out = run_accept(env, logits, draft)
    assert a.tolist() == a_ref.tolist()
    assert out.tolist() == out_ref.tolist()


@pytest.mark.parametrize("V", [24, 37, 4096 + 16])
def test_accept_ties_signed_zeros_and_infinities(env, V):
    """Small-integer logits (every row has many equal maxima), rows of -inf with one
    finite value, rows mixing -0 and +0, the maximum in the first and in the last slot."""
    rng = np.random.default_rng(V)
    Bn, gamma = 12, 3
    logits = rng.integers(-2, 3, (Bn, gamma + 1, V)).astype(np.float16)
    logits[1, :, :] = -np.inf
    logits[1, np.arange(gamma + 1), [V - 1, 0, V // 2, 3]] = [-65504.0, -1.0, 0.0, 65504.0]
    logits[2, 0, :] = 0.0
    logits[2, 0, ::2] = -0.0                      # -0 at index 0 ties with +0 at index 1: index 0 wins
    logits[3, :, :] = np.float16(-3.0)
    logits[3, :, V - 1] = np.float16(-2.998)      # strict maximum in the very last slot
    logits[4, :, :] = np.inf                      # all equal: index 0
    logits[5, 1, :] = np.float16(6.1e-5)          # subnormal neighbourhood
    logits[5, 1, 5] = np.float16(6.2e-5)
    draft = np.array([[acc.top1(logits[b, j]) for j in range(gamma)] for b in range(Bn)], dtype=np.int32)
    draft[6:, 1] = (draft[6:, 1] + 1) % V         # rejection at the second draft
    draft[9:, 0] = (draft[9:, 0] + 1) % V         # ... and at the first
    a_ref, out_ref = acc.greedy_accept(logits, draft)
    a, out = run_accept(env, logits, draft)
    assert a.tolist() == a_ref.tolist()
    assert out.tolist() == out_ref.tolist()
    assert a_ref[:6].tolist() == [3] * 6 and a_ref[6:9].tolist() == [1] * 3 and a_ref[9:].tolist() == [0] * 3


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_accept_benchmark_configuration(env, config):
    """Full size (the launch the benchmark times).  The pure-Python oracle walks a
    sample of the sequences; for all of them the result is checked against the
    planted greedy tokens of the input recipe and against np.argmax."""
    logits, draft, planted = synth.accept_inputs(config)
    Bn, rows, V = logits.shape
    gamma = rows - 1
    a, out = run_accept(env, logits, draft)
    sample = sorted(set(np.linspace(0, Bn - 1, 6).astype(int).tolist()))
    a_ref, out_ref = acc.greedy_accept(logits[sample], draft[sample])
    assert a[sample].tolist() == a_ref.tolist()
    assert out[sample].tolist() == out_ref.tolist()
    greedy = np.argmax(logits, axis=2)
    assert (greedy == planted).all()
    eq = np.cumprod((greedy[:, :gamma] == draft).astype(np.int64), axis=1).sum(axis=1)
    assert a.tolist() == eq.tolist()
    assert 0 < eq.sum() < Bn * gamma or Bn * gamma < 8          # the recipe mixes acceptances and rejections
    for b in range(Bn):
        n = int(a[b])
        assert out[b, :n].tolist() == draft[b, :n].tolist() and out[b, n] == greedy[b, n] and (out[b, n + 1:] == -1).all()


def test_accept_is_deterministic_and_reuses_its_workspace(env):
    torch, B = env
    logits, draft, _ = synth.accept_case(7, 16, 3, 32000)
    lg, dr = dev(torch, logits), dev(torch, draft)
    ws = torch.full((B.accept_workspace_bytes(16, 3, 32000),), 0xA5, dtype=torch.uint8, device="cuda")   # dirty scratch
    n1, o1 = B.greedy_accept(lg, dr, workspace=ws)
    n2, o2 = B.greedy_accept(lg, dr, workspace=ws)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        n3, o3 = B.greedy_accept(lg, dr)
    torch.cuda.synchronize()
    a_ref, out_ref = acc.greedy_accept(logits, draft)
    for n, o in ((n1, o1), (n2, o2), (n3, o3)):
        assert n.cpu().numpy().tolist() == a_ref.tolist() and o.cpu().numpy().tolist() == out_ref.tolist()


@pytest.mark.parametrize("Bn,gamma,S,D", [(1, 1, 4, 8), (4, 3, 12, 128), (8, 3, 2048, 4096), (5, 5, 64, 1032), (3, 2, 3, 16)])
def test_kv_overwrite_matches_oracle(env, Bn, gamma, S, D):
    torch, B = env
    rng = np.random.default_rng(Bn * 1000 + S)
    cache = rng.standard_normal((Bn, S, D)).astype(np.float16)
    kv = rng.standard_normal((Bn, gamma + 1, D)).astype(np.float16)
    a = rng.integers(0, gamma + 1, Bn).astype(np.int32)
    pos = rng.integers(0, S, Bn).astype(np.int32)
    pos[0] = S - 1                                   # runs off the end unless nothing but row 0 is copied
    if Bn > 1:
        pos[1], a[1] = 0, gamma                      # everything accepted at the start of the cache
    ref = acc.kv_overwrite(cache, kv, a, pos)
    guard = np.float16(123.0)
    buf = torch.full((Bn * S * D + 64,), float(guard), dtype=torch.float16, device="cuda")
    c = buf[32:32 + Bn * S * D].view(Bn, S, D)
    c.copy_(dev(torch, cache))
    B.kv_overwrite(c, dev(torch, kv), dev(torch, a), dev(torch, pos))
    torch.cuda.synchronize()
    assert c.cpu().numpy().tobytes() == ref.tobytes()
    assert (buf[:32] == float(guard)).all() and (buf[-32:] == float(guard)).all()


def test_kv_overwrite_clamps_bad_counts_and_skips_rows_outside_the_cache(env):
    torch, B = env
    Bn, gamma, S, D = 4, 3, 8, 64
    rng = np.random.default_rng(1)
    cache = rng.standard_normal((Bn, S, D)).astype(np.float16)
    kv = rng.standard_normal((Bn, gamma + 1, D)).astype(np.float16)
    a = np.array([99, -5, 2, 3], dtype=np.int32)     # out of range on both sides
    pos = np.array([0, 4, -1, 6], dtype=np.int32)    # negative start, and a tail past the end
    ref = acc.kv_overwrite(cache, kv, np.clip(a, 0, gamma), pos)
    c = dev(torch, cache)
    B.kv_overwrite(c, dev(torch, kv), dev(torch, a), dev(torch, pos))
    torch.cuda.synchronize()
    assert c.cpu().numpy().tobytes() == ref.tobytes()


def test_accept_then_overwrite_pipeline(env):
    """The two steps chained on the device, n_accept never leaving it."""
    torch, B = env
    logits, draft, _ = synth.accept_inputs(2)
    Bn, rows, V = logits.shape
    gamma, S, D = rows - 1, 256, 1024
    rng = np.random.default_rng(2)
    cache = rng.standard_normal((Bn, S, D)).astype(np.float16)
    kv = rng.standard_normal((Bn, rows, D)).astype(np.float16)
    pos = rng.integers(0, S - rows, Bn).astype(np.int32)
    n, out = B.greedy_accept(dev(torch, logits), dev(torch, draft))
    c = dev(torch, cache)
    B.kv_overwrite(c, dev(torch, kv), n, dev(torch, pos))
    torch.cuda.synchronize()
    a_ref, _ = acc.greedy_accept(logits, draft)
    assert c.cpu().numpy().tobytes() == acc.kv_overwrite(cache, kv, a_ref, pos).tobytes()
