"""The largest arena the planner accepts (just under 2^33 elements, 34 GB per fp32 buffer), shards of
the largest size it allows (2^30 elements), packed offsets beyond 2^32: every element of send, residual and dense
result is checked on the device, shard by shard, against values that are exact by
construction (small integers, c = 1, N = 2), with the layout taken from the oracle's
planner and filter.  The oracle's element loops are not run at this size (17 GB per
buffer); their arithmetic is covered by the other parity tests, the addressing is what
is at stake here."""
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
CHUNK = 1 << 27


@pytest.fixture(scope="module")
def B():
    from paper_2311_04499_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def pattern(lo: int, hi: int, mult: int) -> torch.Tensor:
    """Integers in [-1000, 1000] as fp32, a fixed function of the element index."""
    i = torch.arange(lo, hi, dtype=torch.int64, device=DEV)
    return ((((i * mult) >> 7) % 2001) - 1000).to(torch.float32)


def fill(t: torch.Tensor, mult: int):
    for lo in range(0, t.numel(), CHUNK):
        hi = min(lo + CHUNK, t.numel())
        t[lo:hi] = pattern(lo, hi, mult)


def test_arena_at_the_planner_s_size_limit(B):
    free, _ = torch.cuda.mem_get_info()
    if free < 170 << 30:
        pytest.skip("needs about 150 GB of device memory")
    S, K, N = 1 << 30, 2, 2
    D = (1 << 33) - (1 << 20) + 12                        # eight shards, the last one short
    with pytest.raises(B.CovapError):
        B.covap_plan([1 << 33, 1], S, K)                   # one element past the limit
    plan = B.covap_plan([D], S, K)
    tab = oracle.plan_fixed([D], S, 1 << 40)
    assert plan.total_elems == D > 1 << 32 and plan.num_shards == tab.n_shards == 8
    G = torch.empty(D, device=DEV)
    R = torch.empty(D, device=DEV)
    out = torch.empty(D, device=DEV)
    MG, MR, MP = 2654435761, 40503, 2246822519
    fill(G, MG)
    for t in (0, 1):
        sel = [s for s in range(tab.n_shards) if oracle.selected(s, t, K)]
        P = sum(int(tab.len[s]) for s in sel)
        assert plan.packed_elems(t) == P == oracle.packed_elems(tab, K, t)
        stride = (P + 255) // 256 * 256
        recv = torch.empty(N, stride, device=DEV)
        fill(recv[1], MP)
        recv[0].fill_(float("nan"))
        fill(R, MR)
        out.fill_(float("nan"))
        B.covap_compress(plan, t, G, R, recv[0])
        B.covap_decompress(plan, t, recv, out)
        torch.cuda.synchronize()
        poff = 0
        for s in range(tab.n_shards):
            off, ln = int(tab.off[s]), int(tab.len[s])
            assert plan.shard(s)[:2] == (off, ln)
            for lo in range(0, ln, CHUNK):
                hi = min(lo + CHUNK, ln)
                A = pattern(off + lo, off + hi, MG) + pattern(off + lo, off + hi, MR)   # exact
                r = R[off + lo:off + hi]
                o = out[off + lo:off + hi]
                if s in sel:
                    assert torch.equal(recv[0, poff + lo:poff + hi], A), (t, s, lo, "send")
                    assert not r.view(torch.int32).any(), (t, s, lo, "residual of a sent shard")
                    want = (A + pattern(poff + lo, poff + hi, MP)) * 0.5                 # exact
                    assert torch.equal(o, want), (t, s, lo, "dense")
                else:
                    assert torch.equal(r, A), (t, s, lo, "residual")
                    assert not o.view(torch.int32).any(), (t, s, lo, "dense of an unsent shard")
            if s in sel:
                poff += ln
        assert poff == P
        assert torch.isnan(recv[0, P:]).all()                  # nothing written past the payload
        del recv


def upattern(lo: int, hi: int, mult: int, bits: int, shift: int) -> torch.Tensor:
    """Multiples of 2^-23 in [-2^(bits-24), 2^(bits-24)) as fp32, a fixed function of the index."""
    i = torch.arange(lo, hi, dtype=torch.int64, device=DEV)
    v = (((i * mult) >> shift) % (1 << bits)) - (1 << (bits - 1))
    return v.to(torch.float32) * (2.0 ** -23)


def test_topk_at_the_largest_supported_size(B):
    """n just below 2^32 (indices use all 32 bits), k = 0.1 %: count, order, values,
    residual, the magnitude cut and the tie rule, all checked on the device.  The inputs
    are multiples of 2^-23 below 1.01 in magnitude, so A = G + R is exact and magnitudes
    repeat about 250 times each: the threshold always has ties."""
    free, _ = torch.cuda.mem_get_info()
    if free < 90 << 30:
        pytest.skip("needs about 80 GB of device memory")
    n = (1 << 32) - 4
    k = -(-n // 1000)
    MG, MR = 2654435761, 2246822519
    G = torch.empty(n, device=DEV)
    R = torch.empty(n, device=DEV)
    for lo in range(0, n, CHUNK):
        hi = min(lo + CHUNK, n)
        G[lo:hi] = upattern(lo, hi, MG, 24, 5)
        R[lo:hi] = upattern(lo, hi, MR, 16, 9)
    ws = torch.empty(B.topk_workspace_bytes(n), dtype=torch.uint8, device=DEV)
    vals = torch.full((k,), float("nan"), device=DEV)
    idx32 = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    B.topk_compress(G, R, k, vals, idx32, ws)
    torch.cuda.synchronize()
    idx = idx32.to(torch.int64) & 0xffffffff
    assert bool((idx[1:] > idx[:-1]).all()) and int(idx[0]) >= 0 and int(idx[-1]) < n
    assert int(idx[-1]) >= 1 << 31                               # the high half of the index range is in use
    r0_kept = ((((idx * MR) >> 9) % (1 << 16)) - (1 << 15)).to(torch.float32) * (2.0 ** -23)
    A_kept = G[idx] + r0_kept
    assert torch.equal(vals, A_kept)
    T = float(vals.abs().min())
    tie_kept = idx[vals.abs() == T]
    assert tie_kept.numel() > 0
    first_tie_left_behind = n
    for lo in range(0, n, CHUNK):
        hi = min(lo + CHUNK, n)
        A = G[lo:hi] + upattern(lo, hi, MR, 16, 9)
        a, b = torch.searchsorted(idx, torch.tensor([lo, hi], device=DEV)).tolist()
        A[idx[a:b] - lo] = 0.0                                   # what the residual must be
        r = R[lo:hi]
        assert torch.equal(r, A), (lo, "residual")
        mag = r.abs()
        assert float(mag.max()) <= T, (lo, "something larger was left behind")
        left = torch.nonzero(mag == T)
        if left.numel() and first_tie_left_behind == n:
            first_tie_left_behind = lo + int(left[0])
    assert int(tie_kept[-1]) < first_tie_left_behind             # ties: lowest indices first
