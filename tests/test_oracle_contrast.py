"""Pins for the oracle's Random-k, FP16 and sparse/half mean functions (CPU only):
numpy's float16 cast (an independent IEEE implementation) for the conversions,
Algorithm 1's identities, exact conservation on integer data, and numpy
scatter/accumulate routines for the means."""
import numpy as np
import pytest

import oracle


def bits(x):
    return np.ascontiguousarray(x).view(np.uint32)


def test_f16_conversions_against_numpy():
    rng = np.random.default_rng(0)
    pats = np.concatenate([
        rng.integers(0, 2 ** 32, 50_000, dtype=np.uint64).astype(np.uint32),
        # boundaries: zero, smallest subnormal and its halfway points, subnormal/normal
        # edge, largest finite and the overflow threshold, infinities
        np.array([0, 0x80000000, 0x33000000, 0x33000001, 0x32ffffff, 0x33800000, 0x337fffff,
                  0x387fe000, 0x387ff000, 0x38800000, 0x477fe000, 0x477fefff, 0x477ff000,
                  0x47800000, 0x7f800000, 0xff800000, 0x7f7fffff, 0x3c001000, 0x3c003000,
                  0x3c000fff, 0x3c001001], dtype=np.uint32)])
    f = pats.view(np.float32)
    f = f[~np.isnan(f)]
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16(float(x)) for x in f], np.uint16)
    assert np.array_equal(got, want)
    h = np.arange(65536, dtype=np.uint16)
    wide = h.view(np.float16).astype(np.float32)
    back = np.array([oracle.f16_to_f32(int(x)) for x in h], np.float32)
    ok = ~np.isnan(wide)
    assert np.array_equal(bits(back[ok]), bits(wide[ok])) and np.isnan(back[~ok]).all()
    assert (oracle.f32_to_f16(float("nan")) & 0x7fff) > 0x7c00


def test_fp16_compress_identities():
    rng = np.random.default_rng(1)
    n = 10_003
    G = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    G[:6] = [0.0, -0.0, 70000.0, 1e-9, 6.0e-8, -65504.0]
    R0 = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    R = R0.copy()
    out = oracle.fp16_compress(G, R, 0.5)
    A = (G.astype(np.float64) + 0.5 * R0.astype(np.float64)).astype(np.float32)
    with np.errstate(over="ignore"):
        want = A.astype(np.float16)
    assert np.array_equal(out, want.view(np.uint16))
    fin = np.isfinite(want)
    assert np.array_equal(want.astype(np.float32)[fin] + R[fin], A[fin])   # nothing lost
    assert np.all(np.abs(R[fin]) <= np.maximum(np.abs(A[fin]) * 2.0 ** -11, 2.0 ** -25))
    assert np.isinf(R[~fin]).all()                  # overflow to Inf leaves an infinite residual


def test_fp16_conservation_over_steps():
    rng = np.random.default_rng(2)
    n, T = 5000, 9
    R = np.zeros(n, np.float32)
    sent = np.zeros(n, np.float64)
    total = np.zeros(n, np.float64)
    for t in range(T):
        G = rng.integers(-3000, 3001, n).astype(np.float32)        # > 11 bits: fp16 must round
        total += G
        h = oracle.fp16_compress(G, R)
        sent += h.view(np.float16).astype(np.float64)
    assert np.array_equal(sent + R, total)
    assert np.any(R != 0)


def test_fp16_mean_is_left_fold():
    rng = np.random.default_rng(3)
    for N in (1, 2, 3, 7, 64):
        n, stride = 1003, 1008
        rows = (rng.standard_normal((N, stride)) * np.logspace(-2, 2, N)[:, None]).astype(np.float16)
        out = oracle.fp16_mean(rows.view(np.uint16), n)
        acc = rows[0, :n].astype(np.float32)
        for w in range(1, N):
            acc = acc + rows[w, :n].astype(np.float32)
        want = (acc.astype(np.float64) / N).astype(np.float32)
        assert np.array_equal(bits(out), bits(want))


@pytest.mark.parametrize("n,k", [(10, 0), (10, 3), (10, 10), (5000, 50), (1, 1)])
def test_randk_against_numpy(n, k):
    rng = np.random.default_rng(n + k)
    G = rng.standard_normal(n).astype(np.float32)
    R0 = rng.standard_normal(n).astype(np.float32)
    idx = rng.permutation(n)[:k].astype(np.uint32)                 # distinct, any order
    R = R0.copy()
    vals = oracle.randk(G, R, idx, 0.5)
    A = (G.astype(np.float64) + 0.5 * R0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(bits(vals), bits(A[idx]))
    want_R = A.copy()
    want_R[idx] = 0.0
    assert np.array_equal(bits(R), bits(want_R))
    dense = np.zeros(n, np.float32)
    dense[idx] = vals
    assert np.array_equal(dense + R, A)


def test_sparse_mean_against_numpy_accumulate():
    rng = np.random.default_rng(5)
    n, k, stride = 2000, 150, 160
    for N in (1, 2, 5, 8):
        idx = np.stack([np.sort(rng.permutation(n)[:stride]) for _ in range(N)]).astype(np.uint32)
        vals = rng.standard_normal((N, stride)).astype(np.float32)
        out = oracle.sparse_mean(vals, idx, k, n)
        acc = np.zeros(n, np.float32)
        for w in range(N):
            acc[idx[w, :k]] = acc[idx[w, :k]] + vals[w, :k]         # distinct inside a row
        want = acc if N == 1 else (acc.astype(np.float64) / N).astype(np.float32)
        assert np.array_equal(bits(out), bits(want))
        # integer-valued check against an order-free routine
        iv = rng.integers(-50, 51, (N, stride)).astype(np.float32)
        out = oracle.sparse_mean(iv, idx, k, n)
        ref = np.zeros(n, np.float64)
        for w in range(N):
            np.add.at(ref, idx[w, :k], iv[w, :k])
        assert np.allclose(out, ref / N, rtol=1e-7, atol=0)
        touched = np.zeros(n, bool)
        touched[idx[:, :k].ravel()] = True
        assert not out[~touched].any()
