"""topk_compress_static -- the entry point for callers that cannot allocate --
against topk_compress on the same inputs: indices, values and residual bit for
bit, on two calls in a row (the second on a smaller input, so that the shared
built-in workspace still holds the first call's contents), and the size limit."""
import numpy as np
import pytest
import torch

from paper_2311_04499_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    from paper_2311_04499_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def both(B, G, R0, k, c):
    n = G.numel()
    out = []
    for static in (False, True):
        R = R0.clone()
        vals = torch.full((max(k, 1),), float("nan"), device=DEV)
        idx = torch.full((max(k, 1),), -1, dtype=torch.int32, device=DEV)
        if static:
            B.topk_compress_static(G, R, k, vals, idx, ef_coeff=c)
        else:
            ws = torch.empty(B.topk_workspace_bytes(n), dtype=torch.uint8, device=DEV)
            B.topk_compress(G, R, k, vals, idx, ws, ef_coeff=c)
        torch.cuda.synchronize()
        out.append((vals[:k].cpu().numpy().view(np.uint32), idx[:k].cpu().numpy(),
                    R.cpu().numpy().view(np.uint32)))
    return out


def same(a, b, what):
    for x, y, name in zip(a, b, ("values", "indices", "residual")):
        assert np.array_equal(x, y), f"{what}: {name} differ"


def test_static_workspace_matches_caller_workspace_on_two_calls_in_a_row(B):
    assert B.topk_static_max_elems() == 1 << 24
    wl = workloads.scaled_down(workloads.config(5), [3_000_017], 4096)
    # first call: 3 M elements (several thousand tiles, ragged end); second: a smaller,
    # differently shaped input on the workspace the first one left behind
    for n, k, c, seed in ((3_000_017, 3_001, 1.0, 0), (70_001, 701, 0.5, 1)):
        G = workloads.gradient(wl, 0, seed, DEV)[:n].contiguous()
        R0 = workloads.gradient(wl, 1, seed, DEV)[:n].contiguous()
        ref, got = both(B, G, R0, k, c)
        assert len(np.unique(got[1])) == k
        same(got, ref, f"n={n}")


def test_static_workspace_ties_and_general_tail(B):
    """Heavily tied data takes the general tail (full histogram passes, atomically
    accumulated rows): the rows must be reset by each call."""
    rng = np.random.default_rng(5)
    for n, k in ((200_003, 50_000), (20_003, 17)):
        G = torch.from_numpy(rng.integers(-3, 4, n).astype(np.float32)).to(DEV)
        R0 = torch.zeros(n, device=DEV)
        ref, got = both(B, G, R0, k, 1.0)
        same(got, ref, f"ties n={n}")


def test_static_workspace_limit_and_errors(B):
    n = B.topk_static_max_elems() + 1
    G = torch.zeros(n, device=DEV)
    R = torch.zeros(n, device=DEV)
    vals = torch.zeros(16, device=DEV)
    idx = torch.zeros(16, dtype=torch.int32, device=DEV)
    with pytest.raises(B.CovapError) as e:
        B.topk_compress_static(G, R, 8, vals, idx)
    assert e.value.status == 1 and "topk_static_max_elems" in str(e.value)
    with pytest.raises(B.CovapError):
        B.topk_compress_static(G, R, 9, vals, idx, n=8)                 # k > n
    with pytest.raises(B.CovapError) as e:
        B.topk_compress_static(G, R, 1, vals, idx, n=8, dtype=B.COVAP_BF16)
    assert e.value.status == 5
    B.topk_compress_static(G, R, 0, vals, idx, n=0)                     # nothing to do
    # the largest size the entry point takes
    n = B.topk_static_max_elems()
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    G = torch.randn(n, generator=g, device=DEV)
    R0 = torch.randn(n, generator=g, device=DEV)
    ref, got = both(B, G, R0, n // 1000, 1.0)
    same(got, ref, "largest n")


def test_static_workspace_under_hip_graph_replay(B):
    """What the entry point is for: captured once in a HIP graph (capture forbids allocation; the call
    records kernels only, no memset node) and replayed with the program's own eager work and
    synchronisations in between; every replay must give the bits the oracle gives for that step's inputs."""
    import oracle
    n, k = 300_017, 301
    wl = workloads.scaled_down(workloads.config(5), [n], 4096)
    G = torch.empty(n, device=DEV)
    R = torch.zeros(n, device=DEV)
    vals = torch.empty(k, device=DEV)
    idx = torch.empty(k, dtype=torch.int32, device=DEV)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    G.copy_(workloads.gradient(wl, 0, 0, DEV))
    B.topk_compress_static(G, R, k, vals, idx, ef_coeff=0.5)      # first use outside capture: the address look-up
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        B.topk_compress_static(G, R, k, vals, idx, ef_coeff=0.5)
    R.zero_()
    Rc = np.zeros(n, np.float32)
    for t in range(4):
        G.copy_(workloads.gradient(wl, 0, t, DEV))
        torch.cuda.synchronize()
        g.replay()
        other = torch.randn(1000, device=DEV).sum().item()        # eager work between replays
        torch.cuda.synchronize()
        ov, oi = oracle.topk(G.cpu().numpy(), Rc, k, 0.5)
        assert np.array_equal(idx.cpu().numpy().view(np.uint32), oi), f"indices t={t}"
        assert np.array_equal(vals.cpu().numpy().view(np.uint32), ov.view(np.uint32)), f"values t={t}"
        assert np.array_equal(R.cpu().numpy().view(np.uint32), Rc.view(np.uint32)), f"residual t={t}"
        assert other == other
