"""Pins for the oracle's mean after a sum-AllReduce (CPU only).

Sec. II-A aggregates the workers' gradients with AllReduce and averages them; Sec. III-B
keeps AllReduce for COVAP because every worker sends the same shards.  What is left for
each worker after the collective is: divide the one summed payload by N and put it back
where the sent shards live, +0 elsewhere.  The oracle's routine is checked against the
exact quotient rounded once (float64 holds fp32 / N to well over twice 24 bits), against
torch's bf16 cast and numpy's float16, on the packed layout restated here from
Definition 1 (sent shards ascending, each at the next multiple of the alignment), on
signed zeros, infinities, NaN and subnormals, and against the N-row mean on data where
the sum is exact whatever its order.
"""
import numpy as np
import pytest
import torch

import oracle


def bits(x):
    x = np.ascontiguousarray(x)
    return x.view(np.uint32 if x.itemsize == 4 else np.uint16)


def layout(tab, I, t):
    """Arena position -> packed position for every sent element, from Definition 1 and the
    packing rule alone; -1 where nothing is sent; -2 in arena padding."""
    where = np.full(tab.D, -2, np.int64)
    p = 0
    for s in range(tab.n_shards):
        o, l = int(tab.off[s]), int(tab.len[s])
        if (s + t) % I == 0:
            p = -(-p // tab.align) * tab.align
            where[o:o + l] = p + np.arange(l)
            p += l
        else:
            where[o:o + l] = -1
    return where, p


def expected(where, summed, N, prefill, quotient):
    out = prefill.copy()
    sent = where >= 0
    out[sent] = quotient(summed[where[sent]], N)
    out[where == -1] = 0
    return out


TABLES = [
    ("fixed", dict(numel=[1000, 37, 5000, 1], S=256, cap=1 << 30), 3),
    ("fixed", dict(numel=[10], S=4, cap=1 << 30), 2),
    ("fixed", dict(numel=[5], S=8, cap=1 << 30), 3),
    ("fixed", dict(numel=[300_000, 12_345], S=8192, cap=100_000), 5),
    ("median", dict(numel=[1003, 2001, 30007, 5, 4099, 17, 90001, 3], cap=5000, ref=0, align=4), 3),
    ("median", dict(numel=[41011, 167813, 1074805, 70794, 76697, 5551], cap=1, ref=55903, align=256), 4),
]


def table(kind, kw, I):
    if kind == "fixed":
        return oracle.plan_fixed(kw["numel"], kw["S"], kw["cap"])
    return oracle.plan_median(kw["numel"], kw["cap"], I, kw["ref"], kw["align"])


def q_f32(x, N):
    return (x.astype(np.float64) / N).astype(np.float32)


def q_bf16(x, N):
    f = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).float()
    return (f / N).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def q_pay16(x, N):
    return (x.view(np.float16).astype(np.float64) / N).astype(np.float32)


SPECIALS = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -3e-45, 1.1754942e-38, 1e-40, 3.4e38, -3.4e38,
                     1.0, -1.0, 3.0, 65504.0, 6e-8], np.float32)


def payload(rng, P, kind):
    x = (rng.standard_normal(P + 8) * 10.0 ** rng.integers(-6, 6, P + 8)).astype(np.float32)
    x[:min(P, SPECIALS.size)] = SPECIALS[:min(P, SPECIALS.size)]
    if kind == "f32":
        return x
    if kind == "bf16":
        with np.errstate(invalid="ignore"):
            return torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    with np.errstate(over="ignore"):
        return x.astype(np.float16).view(np.uint16).copy()


@pytest.mark.parametrize("kind,kw,I", TABLES)
@pytest.mark.parametrize("form", ["f32", "bf16", "pay16"])
def test_quotient_rounded_once_at_the_sent_positions_zero_elsewhere(kind, kw, I, form):
    tab = table(kind, kw, I)
    rng = np.random.default_rng(31)
    out_t = np.uint16 if form == "bf16" else np.float32
    quotient = dict(f32=q_f32, bf16=q_bf16, pay16=q_pay16)[form]
    for t in list(range(I + 1)) + [10 ** 12 + 5]:
        where, P = layout(tab, I, t)
        assert P == oracle.packed_elems(tab, I, t)
        for N in (1, 2, 3, 7, 64, 100):
            summed = payload(rng, P, form)
            pre = np.full(tab.D, 0x7fc1 if form == "bf16" else np.nan, out_t)
            out = pre.copy()
            oracle.unpack_mean(tab, I, t, summed, N, out)
            want = expected(where, summed, N, pre, quotient)
            assert np.array_equal(bits(out), bits(want)), (t, N)
            # the same call bucket by bucket, and on threads over runs of shards
            out_b = pre.copy()
            for b in range(tab.n_buckets):
                oracle.unpack_mean(tab, I, t, summed, N, out_b, bucket=b)
            assert np.array_equal(bits(out_b), bits(want))
            out_th = pre.copy()
            oracle.unpack_mean(tab, I, t, summed, N, out_th, threads=3)
            assert np.array_equal(bits(out_th), bits(want))


def test_one_worker_returns_the_payload_and_powers_of_two_scale_exactly():
    tab = oracle.plan_fixed([4096 + 3], 256, 1 << 30)
    I, t = 2, 1
    where, P = layout(tab, I, t)
    rng = np.random.default_rng(5)
    x = rng.standard_normal(P).astype(np.float32)
    x[:4] = [0.0, -0.0, 1e-45, -3.4e38]
    sent = where >= 0
    out = np.full(tab.D, np.nan, np.float32)
    oracle.unpack_mean(tab, I, t, x, 1, out)
    assert np.array_equal(bits(out[sent]), bits(x[where[sent]]))
    for e in (1, 3, 6):
        oracle.unpack_mean(tab, I, t, x[4:].copy(), 1 << e, out)   # normal numbers only: ldexp is exact
        src = where[sent]
        ok = src < P - 4
        assert np.array_equal(out[sent][ok], np.ldexp(x[4:][src[ok]], -e))
    # the sign of a zero survives the division
    z = np.zeros(P, np.float32)
    z[::2] = -0.0
    oracle.unpack_mean(tab, I, t, z, 64, out)
    assert np.array_equal(bits(out[sent]), bits(z[where[sent]]))
    assert not bits(out[~sent]).any()


@pytest.mark.parametrize("N", [2, 3, 8, 64])
def test_equals_the_row_mean_when_the_sum_is_exact(N):
    """Integer-valued payloads: the sum of N rows is exact in fp32 whatever the order the
    collective adds them in, so dividing that sum must give what the N-row mean gives."""
    tab = oracle.plan_median([1003, 2001, 30007, 5, 4099, 17], 5000, 3, 0, 4)
    I = 3
    rng = np.random.default_rng(17)
    for t in range(I):
        P = oracle.packed_elems(tab, I, t)
        rows = rng.integers(-1000, 1000, (N, P + 4)).astype(np.float32)
        a = np.zeros(tab.D, np.float32)
        b = np.ones(tab.D, np.float32)
        oracle.decompress(tab, I, t, rows, a)
        summed = rows.astype(np.float64).sum(axis=0).astype(np.float32)
        oracle.unpack_mean(tab, I, t, summed, N, b)
        covered = layout(tab, I, t)[0] != -2
        assert np.array_equal(bits(a[covered]), bits(b[covered]))
        assert np.all(b[~covered] == 1)                             # arena padding is never written


def test_identical_workers_round_trip_through_compress():
    """N = 4 identical workers: the collective's sum is 4 x payload (exact), and the mean
    put back in place is the filtered gradient of Definition 1."""
    tab = oracle.plan_fixed([5000, 300], 512, 1 << 30)
    I, N = 3, 4
    G = np.random.default_rng(4).standard_normal(tab.D).astype(np.float32)
    for t in range(I):
        R = np.zeros(tab.D, np.float32)
        send = np.zeros(oracle.packed_elems(tab, I, t), np.float32)
        oracle.compress(tab, I, t, G, R, send)
        out = np.full(tab.D, np.nan, np.float32)
        oracle.unpack_mean(tab, I, t, send * np.float32(N), N, out)
        assert np.array_equal(out + R, G)
        assert not bits(out[R != 0]).any()                          # unsent: +0 here, the value stays in R
