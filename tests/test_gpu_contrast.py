"""GPU parity of the Random-k / FP16 contrast kernels and the sparse / half
means against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_04499_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    from paper_2311_04499_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def u32(a):
    return np.ascontiguousarray(a).view(np.uint32)


def same(got, want, what):
    if got.dtype == np.float32:
        ng, nw = np.isnan(got), np.isnan(want)
        assert np.array_equal(ng, nw), what
        assert np.array_equal(u32(got)[~ng], u32(want)[~nw]), what
    else:
        assert np.array_equal(got, want), what


SIZES = [1, 3, 4, 7, 8, 9, 63, 64, 65, 1023, 4099, 262_147, 3_000_001]


@pytest.mark.parametrize("n", SIZES)
def test_fp16_compress_and_mean(B, n):
    wl = workloads.scaled_down(workloads.config(5), [n], 4096)
    R = torch.zeros(n, device=DEV)
    Rc = np.zeros(n, np.float32)
    N = 5
    stride = (n + 7) // 8 * 8
    recv = torch.zeros(N, stride, dtype=torch.float16, device=DEV)
    for t in range(3):
        G = workloads.gradient(wl, 0, t, DEV)
        if n > 8:
            G[:8] = torch.tensor([0.0, -0.0, 70000.0, 1e-9, 6.0e-8, -65504.0, 65520.0, 3e-5], device=DEV)
        B.fp16_compress(G, R, recv[0], ef_coeff=0.5, n=n)
        hc = oracle.fp16_compress(G.cpu().numpy(), Rc, 0.5)
        torch.cuda.synchronize()
        same(recv[0, :n].cpu().view(torch.int16).numpy().view(np.uint16), hc, f"payload t={t}")
        same(R.cpu().numpy(), Rc, f"residual t={t}")
        R.nan_to_num_(posinf=0.0, neginf=0.0); np.nan_to_num(Rc, copy=False, posinf=0.0, neginf=0.0)
        recv[1:] = (workloads.payload_rows(wl, N - 1, stride, t, DEV)).to(torch.float16)
        out = torch.full((n,), float("nan"), device=DEV)
        B.fp16_decompress(recv, out, n=n)
        recv_c = recv.cpu().view(torch.int16).numpy().view(np.uint16).copy()
        recv_c[0, :n] = hc                                   # the oracle averages its own payload, not the GPU's
        want = oracle.fp16_mean(recv_c, n)
        torch.cuda.synchronize()
        same(out.cpu().numpy(), want, f"mean t={t}")


@pytest.mark.parametrize("N", [1, 2, 3, 7, 64])
def test_fp16_mean_worker_counts(B, N):
    n, stride = 70_003, 70_008
    g = torch.Generator(device=DEV).manual_seed(N)
    recv = (torch.randn(N, stride, generator=g, device=DEV) * 1e-2).to(torch.float16)
    out = torch.empty(n, device=DEV)
    B.fp16_decompress(recv, out, n=n)
    want = oracle.fp16_mean(recv.cpu().view(torch.int16).numpy().view(np.uint16), n)
    torch.cuda.synchronize()
    same(out.cpu().numpy(), want, "mean")


@pytest.mark.parametrize("n", SIZES)
def test_randk_and_sparse_mean(B, n):
    wl = workloads.scaled_down(workloads.config(5), [n], 4096)
    k = max(1, n // 100) if n > 3 else n
    N = 4
    R = torch.zeros(n, device=DEV)
    Rc = np.zeros(n, np.float32)
    gen = torch.Generator().manual_seed(n)
    vals_all = torch.zeros(N, k, device=DEV)
    idx_all = torch.zeros(N, k, dtype=torch.int32, device=DEV)
    for t in range(3):
        G = workloads.gradient(wl, 0, t, DEV)
        idx = torch.randperm(n, generator=gen)[:k].sort().values.to(torch.int32)
        idx_d = idx.to(DEV)
        vals = torch.full((k,), float("nan"), device=DEV)
        B.randk_compress(G, R, idx_d, vals, ef_coeff=0.5)
        vc = oracle.randk(G.cpu().numpy(), Rc, idx.numpy().view(np.uint32), 0.5)
        torch.cuda.synchronize()
        same(vals.cpu().numpy(), vc, f"vals t={t}")
        same(R.cpu().numpy(), Rc, f"residual t={t}")
    # N sparse payloads with overlapping supports -> dense mean
    for w in range(N):
        idx_all[w] = torch.randperm(n, generator=gen)[:k].sort().values.to(torch.int32).to(DEV)
        vals_all[w] = torch.randn(k, generator=gen).to(DEV)
    for workers in (1, 3, N):
        out = torch.full((n,), float("nan"), device=DEV)
        B.sparse_decompress(vals_all, idx_all, out, n_workers=workers)
        want = oracle.sparse_mean(vals_all[:workers].cpu().numpy().copy(),
                                  idx_all[:workers].cpu().numpy().view(np.uint32).copy(), k, n)
        torch.cuda.synchronize()
        same(out.cpu().numpy(), want, f"sparse mean N={workers}")
        out2 = torch.full((n,), float("nan"), device=DEV)         # rows ascend: the one-pass form applies
        B.sparse_decompress_sorted(vals_all, idx_all, out2, n_workers=workers)
        torch.cuda.synchronize()
        same(out2.cpu().numpy(), want, f"sorted sparse mean N={workers}")


def test_topk_payloads_round_trip_through_sparse_mean(B):
    """topk_compress on N workers, then sparse_decompress: against the oracle's two steps."""
    n, N = 500_003, 3
    k = -(-n // 1000)
    wl = workloads.scaled_down(workloads.config(5), [n], 4096)
    ws = torch.empty(B.topk_workspace_bytes(n), dtype=torch.uint8, device=DEV)
    vals = torch.zeros(N, k, device=DEV)
    idx = torch.zeros(N, k, dtype=torch.int32, device=DEV)
    vc, ic = np.zeros((N, k), np.float32), np.zeros((N, k), np.uint32)
    for w in range(N):
        G = workloads.gradient(wl, w, 0, DEV)
        R = torch.zeros(n, device=DEV)
        B.topk_compress(G, R, k, vals[w], idx[w], ws)
        vc[w], ic[w] = oracle.topk(G.cpu().numpy(), np.zeros(n, np.float32), k)
    out = torch.empty(n, device=DEV)
    B.sparse_decompress(vals, idx, out)
    torch.cuda.synchronize()
    same(idx.cpu().numpy().view(np.uint32), ic, "idx")
    same(out.cpu().numpy(), oracle.sparse_mean(vc, ic, k, n), "dense mean")
    out.fill_(float("nan"))
    B.sparse_decompress_sorted(vals, idx, out)
    torch.cuda.synchronize()
    same(out.cpu().numpy(), oracle.sparse_mean(vc, ic, k, n), "dense mean, one pass")


@pytest.mark.parametrize("n,k,N,kind", [
    (100_003, 3_000, 64, "uniform"),        # every lane has a row; N = 2^6 takes the scaling path
    (100_003, 3_000, 65, "uniform"),        # more rows than lanes: handed to the per-worker form
    (70_001, 5_000, 5, "clustered"),        # hundreds of entries of one row in one tile
    (8_192 * 3, 8_192 * 3, 3, "uniform"),   # k = n: every element of every row
    (20_000, 0, 4, "uniform"),              # empty payloads
    (5, 2, 7, "uniform"),
    (300_007, 2_000, 32, "subnormal"),      # sums that are subnormal or cancel to zero
    (300_007, 2_000, 16, "same_support"),   # every row hits the same elements: the order of the adds matters
])
def test_sorted_sparse_mean_shapes(B, n, k, N, kind):
    rng = np.random.default_rng(n + k + N)
    ic = np.zeros((N, max(k, 1)), np.uint32)
    for w in range(N):
        if kind == "clustered":                                  # all of the row inside two short ranges
            pool = np.concatenate([np.arange(9_000, 12_000), np.arange(60_000, 63_000)])
            ic[w, :k] = np.sort(rng.choice(pool, k, replace=False))
        elif kind == "same_support" and w > 0:
            ic[w] = ic[0]
        elif k:
            ic[w, :k] = np.sort(rng.choice(n if kind != "subnormal" else 4_000, k, replace=False))
    vc = rng.standard_normal((N, max(k, 1))).astype(np.float32)
    if kind == "subnormal":
        vc = (vc * np.float32(1e-38)).astype(np.float32)         # partial sums cross the subnormal range
    if kind == "same_support":
        vc = (vc * (10.0 ** rng.integers(-3, 4, vc.shape))).astype(np.float32)   # rounding depends on the order
    vals = torch.from_numpy(vc).to(DEV)
    idx = torch.from_numpy(ic.view(np.int32)).to(DEV)
    out = torch.full((n,), float("nan"), device=DEV)
    B.sparse_decompress_sorted(vals, idx, out, k=k, n_workers=N)
    torch.cuda.synchronize()
    same(out.cpu().numpy(), oracle.sparse_mean(vc, ic, k, n), "dense mean")


@pytest.mark.parametrize("n,N", [(30_000_017, 64), (12_345_678, 20), (9_000_001, 9), (20_000_000, 32)])
def test_sorted_sparse_mean_long_runs(B, n, N):
    """Arenas of thousands of tiles: a workgroup then walks a run of many tiles, the four tile buffers are
    reused phase after phase and the cursors and prefetched windows are carried along.  Rows mix a spread part
    (one entry per cell), a stretch where every row hits the same elements (the order of the adds matters) and a
    dense cluster (hundreds of entries of a row in one tile)."""
    rng = np.random.default_rng(n + N)
    cell = 1_000
    k_spread = n // cell
    shared = np.sort(rng.choice(np.arange(n // 3, n // 3 + 200_000), 3_000, replace=False)).astype(np.uint32)
    rows_i, rows_v = [], []
    for w in range(N):
        spread = (np.arange(k_spread, dtype=np.int64) * cell + rng.integers(0, cell, k_spread)).astype(np.uint32)
        lo = n // 2 + 50_000 * (w % 3)
        cluster = (lo + np.sort(rng.choice(20_000, 2_500, replace=False))).astype(np.uint32)
        i = np.unique(np.concatenate([spread, shared, cluster]))
        rows_i.append(i)
    k = min(len(i) for i in rows_i)
    ic = np.stack([np.sort(rng.choice(i, k, replace=False)) if len(i) > k else i for i in rows_i]).astype(np.uint32)
    vc = (rng.standard_normal((N, k)) * 10.0 ** rng.integers(-3, 4, (N, k))).astype(np.float32)
    vals = torch.from_numpy(vc).to(DEV)
    idx = torch.from_numpy(ic.view(np.int32)).to(DEV)
    out = torch.full((n,), float("nan"), device=DEV)
    B.sparse_decompress_sorted(vals, idx, out, k=k, n_workers=N)
    torch.cuda.synchronize()
    same(out.cpu().numpy(), oracle.sparse_mean(vc, ic, k, n), f"dense mean n={n} N={N}")
    out2 = torch.full((n,), float("nan"), device=DEV)
    B.sparse_decompress(vals, idx, out2, k=k, n_workers=N)             # the per-worker form: the same bits
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))


def test_argument_errors(B):
    G = torch.zeros(100, device=DEV)
    R = torch.zeros(100, device=DEV)
    h = torch.zeros(104, dtype=torch.float16, device=DEV)
    idx = torch.zeros(10, dtype=torch.int32, device=DEV)
    v = torch.zeros(10, device=DEV)
    with pytest.raises(B.CovapError):
        B.randk_compress(G, R, torch.zeros(101, dtype=torch.int32, device=DEV), torch.zeros(101, device=DEV), k=101)
    with pytest.raises(ValueError):                                  # the binding refuses short buffers itself
        B.randk_compress(G, R, idx, v, k=11)
    with pytest.raises(B.CovapError):
        B.fp16_compress(G[1:], R, h)
    with pytest.raises(B.CovapError):
        B.fp16_decompress(torch.zeros(208, dtype=torch.float16, device=DEV), G, n=100, n_workers=2, stride_elems=50)
    with pytest.raises(B.CovapError):
        B.sparse_decompress(v.view(1, 10), idx.view(1, 10), G, n_workers=0)
    torch.cuda.synchronize()
