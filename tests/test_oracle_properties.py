"""Randomised properties of the oracle (CPU only, hypothesis): the guarantees that the
filter of Definition 1 and Algorithm 1 give for ANY shard layout, interval, step and data,
stated directly from the paper's definitions with independent index arithmetic."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle

layouts = st.tuples(
    st.lists(st.integers(1, 3000), min_size=1, max_size=6),      # tensor sizes
    st.sampled_from([4, 8, 64, 100, 256, 1024]),                 # shard size
    st.integers(1, 9),                                           # interval I
    st.integers(0, 10_000),                                      # first step
)


@settings(max_examples=60, deadline=None)
@given(layouts)
def test_every_shard_goes_out_exactly_once_per_interval(layout):
    numel, S, I, t0 = layout
    tab = oracle.plan_fixed(numel, S, 1 << 30)
    D = sum(numel)
    assert tab.D == D and int(tab.len.sum()) == D
    assert np.array_equal(tab.off, np.arange(tab.n_shards) * S)
    times = np.zeros(tab.n_shards, int)
    total = 0
    for t in range(t0, t0 + I):
        sel = [s for s in range(tab.n_shards) if oracle.selected(s, t, I)]
        assert sel == [s for s in range(tab.n_shards) if (s + t) % I == 0]      # Definition 1, 0-based
        times[sel] += 1
        P = oracle.packed_elems(tab, I, t)
        assert P == sum(int(tab.len[s]) for s in sel)
        total += P
    assert np.all(times == 1) and total == D


@settings(max_examples=40, deadline=None)
@given(layouts, st.integers(0, 2 ** 32 - 1), st.sampled_from([1.0, 0.5, 0.3, 0.0]))
def test_nothing_is_lost_and_nothing_is_invented(layout, seed, c):
    """One step of Algorithm 1 on arbitrary data: every element of A = fma(c, R, G) ends up
    in exactly one place, the payload (sent shards, in order) or the residual, bit for bit;
    the other place holds +0.  Averaging N identical payloads returns the payload."""
    numel, S, I, t = layout
    tab = oracle.plan_fixed(numel, S, 1 << 30)
    D = tab.D
    rng = np.random.default_rng(seed)
    G = (rng.standard_normal(D) * 10.0 ** rng.integers(-6, 6, D)).astype(np.float32)
    R = (rng.standard_normal(D) * 10.0 ** rng.integers(-6, 6, D)).astype(np.float32)
    # c*r is exact in float64 (24 x 24 bits); the sum is then rounded to float64 and to float32,
    # which differs from one rounding only on a tie that needs more than 53 bits (about 2^-29
    # per element): the same evaluation the fixed-case pins use
    A = (np.float64(np.float32(c)) * R.astype(np.float64) + G.astype(np.float64)).astype(np.float32)
    mask = np.zeros(D, bool)
    for s in range(tab.n_shards):
        if (s + t) % I == 0:
            mask[int(tab.off[s]):int(tab.off[s] + tab.len[s])] = True
    send = np.full(D + 4, np.float32(7.0), np.float32)
    n = oracle.compress(tab, I, t, G, R, send, c)
    assert n == int(mask.sum())
    assert np.array_equal(send[:n].view(np.uint32), A[mask].view(np.uint32))      # the payload, in shard order
    assert np.all(send[n:] == np.float32(7.0))                                    # nothing written past it
    assert not R[mask].view(np.uint32).any()                                      # +0 where sent
    assert np.array_equal(R[~mask].view(np.uint32), A[~mask].view(np.uint32))     # A where kept
    N = 3
    recv = np.tile(send[None, :n + (-n) % 4 + 4], (N, 1)).copy()
    out = np.full(D, np.float32(9.0), np.float32)
    oracle.decompress(tab, I, t, recv, out)
    assert not out[~mask].view(np.uint32).any()
    want = ((send[:n] + send[:n]) + send[:n]) / np.float32(3.0)
    assert np.array_equal(out[mask].view(np.uint32), want.astype(np.float32).view(np.uint32))


@settings(max_examples=40, deadline=None)
@given(st.lists(st.integers(1, 5000), min_size=1, max_size=12), st.integers(1, 12), st.integers(4, 4000))
def test_median_plan_is_a_partition_with_aligned_pieces(layers, I, cap):
    for align in (4, 8, 256):
        tab = oracle.plan_median(layers, cap, I, 0, align)
        ends = tab.off + tab.len
        assert np.all(tab.len > 0) and np.all(tab.off[1:] >= ends[:-1])          # ordered, disjoint
        assert int(tab.len.sum()) == sum(layers)                                  # covers every layer element
        assert np.all(tab.off % align == 0)                                       # every piece starts aligned
        first_of_bucket = np.r_[True, tab.bucket[1:] != tab.bucket[:-1]]
        assert np.all(tab.off[first_of_bucket] % align == 0)                      # buckets start aligned
        assert np.all((tab.off[~first_of_bucket] == ends[:-1][~first_of_bucket[1:]]))  # pieces of a bucket are contiguous
        for b in range(tab.n_buckets):
            assert int((tab.bucket == b).sum()) <= max(I, 1)                      # never more than I pieces
