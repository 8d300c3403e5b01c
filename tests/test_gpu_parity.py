"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element and bit for bit, on the same seeded inputs.

Bar: selection, packing positions, error feedback, residuals and the N-way mean
are all bit-exact (the mean keeps the oracle's summation order w = 0..N-1 and
uses IEEE division).  The only exception is the payload of a NaN, which
hardware and libm may propagate differently: NaN positions must coincide.
"""
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
    binding.lib()                      # raises if the HIP library is not built
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def bits(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.float32:
        return a.view(np.uint32)
    return a


def assert_same(got: np.ndarray, want: np.ndarray, what: str):
    gb, wb = bits(got), bits(want)
    if np.array_equal(gb, wb):
        return
    if got.dtype == np.float32:
        nan_g, nan_w = np.isnan(got), np.isnan(want)
        if np.array_equal(nan_g, nan_w) and np.array_equal(gb[~nan_g], wb[~nan_w]):
            return
    bad = np.nonzero(gb != wb)[0]
    raise AssertionError(f"{what}: {bad.size} of {gb.size} elements differ, first at {bad[0]}: "
                         f"got {got[bad[0]]!r} want {want[bad[0]]!r}")


def make_plans(B, numel, S, K, dtype=torch.float32, cap_bytes=25 << 20):
    code = B.COVAP_F32 if dtype == torch.float32 else B.COVAP_BF16
    esz = 4 if dtype == torch.float32 else 2
    plan = B.covap_plan(numel, S, K, dtype=code, bucket_cap_bytes=cap_bytes)
    tab = oracle.plan_fixed(numel, S, max(1, cap_bytes // esz))
    assert plan.total_elems == tab.D and plan.num_shards == tab.n_shards
    assert plan.num_buckets == tab.n_buckets
    return plan, tab


def make_median_plans(B, numel, K, dtype=torch.float32, cap_bytes=25 << 20, ref=0):
    code = B.COVAP_F32 if dtype == torch.float32 else B.COVAP_BF16
    esz = 4 if dtype == torch.float32 else 2
    plan = B.covap_plan(numel, 0, K, dtype=code, bucket_cap_bytes=cap_bytes,
                        mode=B.COVAP_SHARD_MEDIAN, ref_elems=ref)
    tab = oracle.plan_median(numel, max(1, cap_bytes // esz), K, ref, 1024 // esz)   # 1 KiB alignment unit
    assert plan.total_elems == tab.D and plan.num_shards == tab.n_shards
    assert plan.num_buckets == tab.n_buckets
    return plan, tab


def run_iterations(B, wl, numel, S, K, N, iters, dtype=torch.float32, c=1.0, per_bucket=False,
                   cap_bytes=25 << 20, slack=0, plans=None, max_workgroups=None):
    """Full-fidelity loop: every one of the N workers compresses its own gradient
    each iteration; their send buffers are the rows handed to decompress.  Both
    sides run the same loop on the same inputs and are compared after every call."""
    plan, tab = plans if plans is not None else make_plans(B, numel, S, K, dtype, cap_bytes)
    D, P = tab.D, plan.packed_elems_max
    epv = 4 if dtype == torch.float32 else 8
    stride = (P + slack + epv - 1) // epv * epv
    np_dt = np.float32 if dtype == torch.float32 else np.uint16
    R_gpu = [torch.zeros(D, dtype=dtype, device=DEV) for _ in range(N)]
    R_cpu = [np.zeros(D, np_dt) for _ in range(N)]
    for t in range(iters):
        assert plan.packed_elems(t) == oracle.packed_elems(tab, K, t)
        assert plan.selected(t) == [s for s in range(tab.n_shards) if oracle.selected(s, t, K)]
        recv_gpu = torch.full((N, stride), float("nan"), dtype=dtype, device=DEV)
        recv_cpu = to_np(recv_gpu)
        buckets = range(tab.n_buckets) if per_bucket else [-1]
        for w in range(N):
            G = workloads.gradient(wl, w, t, DEV, dtype)
            if G.numel() < D:                                   # arena with alignment padding
                G = torch.cat([G, torch.ones(D - G.numel(), dtype=dtype, device=DEV)])
            G = G[:D].contiguous()
            Gn = to_np(G)
            for b in buckets:
                B.covap_compress(plan, t, G, R_gpu[w], recv_gpu[w], ef_coeff=c, bucket=b,
                                 max_workgroups=max_workgroups)
                oracle.compress(tab, K, t, Gn, R_cpu[w], recv_cpu[w], c, bucket=b)
            torch.cuda.synchronize()
            assert_same(to_np(recv_gpu[w]), recv_cpu[w], f"send t={t} w={w}")
            assert_same(to_np(R_gpu[w]), R_cpu[w], f"residual t={t} w={w}")
        out_gpu = torch.full((D,), float("nan"), dtype=dtype, device=DEV)
        out_cpu = to_np(out_gpu)                                # padding elements stay as they were
        for b in buckets:
            B.covap_decompress(plan, t, recv_gpu, out_gpu, bucket=b)
            oracle.decompress(tab, K, t, recv_cpu, out_cpu, bucket=b)
        torch.cuda.synchronize()
        assert_same(to_np(out_gpu), out_cpu, f"dense t={t}")


# ------------------------------------------------------------------ configurations

def test_cfg1_tiny_mlp_full(B):
    wl = workloads.config(1)
    run_iterations(B, wl, wl.numel, wl.shard_elems, wl.K, wl.n_workers, wl.iterations)


@pytest.mark.parametrize("cfg,numel,S", [
    (2, [1_000_003, 64 * 64 * 9, 2048 * 512, 1000], 65536),     # several shards + ragged tail
    (3, [3 * 1048576 + 12328], 1 << 20),
    (4, [768 * 768] * 3 + [3072 * 768, 768, 2], 1 << 18),
    (5, [2 * 1048576 + 404480, 1024], 1 << 20),
])
def test_scaled_configs(B, cfg, numel, S):
    wl = workloads.scaled_down(workloads.config(cfg), numel, S)
    run_iterations(B, wl, numel, S, wl.K, min(wl.n_workers, 8), 2 * wl.K + 1)


@pytest.mark.parametrize("c", [0.25, 0.5, 0.3])
def test_ef_coefficient_sweep(B, c):
    wl = workloads.scaled_down(workloads.config(1), [70_001], 4096)
    run_iterations(B, wl, [70_001], 4096, 3, 2, 7, c=c)


@pytest.mark.parametrize("N", [1, 3, 5, 7, 24, 64])
def test_worker_counts(B, N):
    wl = workloads.scaled_down(workloads.config(1), [40_961], 4096)
    run_iterations(B, wl, [40_961], 4096, 2, N, 3)


@pytest.mark.parametrize("numel,S,K", [
    ([1], 4, 1), ([3], 4, 2), ([4], 4, 4), ([5], 4, 3), ([4095], 4096, 2), ([4097], 4096, 2),
    ([8193], 8, 5), ([100], 1 << 20, 16),                       # fewer shards than K
    ([12_289], 12, 4), ([50_000], 1000, 1), ([65_537], 16384, 7),
])
def test_edge_shapes(B, numel, S, K):
    wl = workloads.scaled_down(workloads.config(1), numel, S)
    run_iterations(B, wl, numel, S, K, 3, 2 * K + 1, slack=5)


def test_per_bucket_calls(B):
    numel = [300_000, 12_345]
    wl = workloads.scaled_down(workloads.config(2), numel, 8192)
    run_iterations(B, wl, numel, 8192, 3, 2, 4, per_bucket=True, cap_bytes=100_000, c=0.5)


@pytest.mark.parametrize("groups", [1, 7, 300, 1_000_000])
def test_bounded_grid_compress(B, groups):
    """covap_compress_bounded: a grid of at most `groups` workgroups walks the tiles; same bits as the
    oracle whatever the bound (one workgroup doing everything, a bound that does not divide the tile
    count, a bound above it), on both shard layouts and element types, whole-arena and per bucket."""
    wl = workloads.scaled_down(workloads.config(1), [100_003], 4096)
    run_iterations(B, wl, [100_003], 4096, 3, 2, 4, max_workgroups=groups, c=0.5)
    run_iterations(B, wl, [9_001, 12_345], 1000, 5, 2, 6, per_bucket=True, cap_bytes=9000, max_workgroups=groups)
    run_iterations(B, wl, [8 * 4096 + 9], 8192, 4, 2, 5, dtype=torch.bfloat16, max_workgroups=groups)
    layers = [1_003, 2_001, 30_007, 5, 4_099, 17, 90_001, 3]
    wl = workloads.scaled_down(workloads.config(3), layers, 4096)
    for dtype in (torch.float32, torch.bfloat16):
        plans = make_median_plans(B, layers, 4, dtype=dtype, cap_bytes=40_000)
        run_iterations(B, wl, layers, 0, 4, 2, 5, dtype=dtype, plans=plans, max_workgroups=groups)
    if groups == 300:
        layers = [2_500_000, 7]                                  # thousands of tiles per workgroup's walk
        wl = workloads.scaled_down(workloads.config(3), layers, 4096)
        plans = make_median_plans(B, layers, 2, cap_bytes=4)
        run_iterations(B, wl, layers, 0, 2, 2, 3, plans=plans, max_workgroups=groups, per_bucket=True)
        with pytest.raises(B.CovapError):
            plan, _ = make_plans(B, [1000], 64, 2)
            z = torch.zeros(1000, device=DEV)
            B.covap_compress(plan, 0, z, torch.zeros_like(z), torch.zeros_like(z), max_workgroups=0)


KNOBS = {"compress_threads": [64, 256], "compress_unroll": [1, 2, 4],
         "decompress_threads": [64, 256], "decompress_tile": [1, 2, 4],
         "decompress_unroll": [1, 2, 4], "nontemporal": [0, 1],
         "decompress_lds_pad": [0, 8192, 24576, 32768, 49152, 6144]}


@pytest.mark.parametrize("key", list(KNOBS))
def test_launch_shape_knobs(B, key):
    """Every launch shape the tuning knobs can select gives the same bits."""
    old = {k: B.covap_tune_get(k) for k in KNOBS}
    try:
        for v in KNOBS[key]:
            B.covap_tune_set(key, v)
            wl = workloads.scaled_down(workloads.config(1), [100_003], 4096)
            run_iterations(B, wl, [100_003], 4096, 3, 5, 4)
            run_iterations(B, wl, [9_001, 12_345], 1000, 5, 3, 6, per_bucket=True, cap_bytes=9000)
            run_iterations(B, wl, [8 * 4096 + 9], 8192, 4, 3, 5, dtype=torch.bfloat16)
    finally:
        for k in old:
            B.covap_tune_set(k, -1)                    # back to never set


def test_largest_launch_shapes_together(B):
    old = {k: B.covap_tune_get(k) for k in KNOBS}
    try:
        for k in KNOBS:
            B.covap_tune_set(k, KNOBS[k][-1])
        wl = workloads.scaled_down(workloads.config(1), [300_007], 16384)
        run_iterations(B, wl, [300_007], 16384, 4, 9, 5)
    finally:
        for k in old:
            B.covap_tune_set(k, -1)                    # back to never set


@pytest.mark.parametrize("numel,S,K,N", [([100_003], 4096, 3, 4), ([7], 8, 2, 3), ([8 * 4096 + 9], 8192, 4, 5),
                                         ([768 * 768, 3072 * 768 + 5], 1 << 18, 6, 32)])
def test_bf16(B, numel, S, K, N):
    wl = workloads.scaled_down(workloads.config(4), numel, S)
    run_iterations(B, wl, numel, S, K, N, 2 * K + 1, dtype=torch.bfloat16, c=0.5)


def test_special_values(B):
    """Signed zeros, infinities, NaN, denormals: same bits as the oracle (NaN
    payload aside), and a sent element leaves residual +0 whatever it was."""
    D, S, K, N = 4096 * 2 + 6, 4096, 2, 3
    plan, tab = make_plans(B, [D], S, K)
    specials = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 1e-39, 3.4e38, -3.4e38,
                         1.17549435e-38, 1.0, -1.0], np.float32)
    rng = np.random.default_rng(0)
    Gn = rng.choice(specials, D).astype(np.float32)
    Rn = rng.choice(specials, D).astype(np.float32)
    for t in range(2):
        G = torch.from_numpy(Gn).to(DEV)
        R = torch.from_numpy(Rn).to(DEV)
        P = plan.packed_elems_max
        stride = (P + 3) // 4 * 4
        send = torch.zeros(stride, device=DEV)
        Rc, sc = Rn.copy(), np.zeros(stride, np.float32)
        B.covap_compress(plan, t, G, R, send, ef_coeff=0.5)
        oracle.compress(tab, K, t, Gn, Rc, sc, 0.5)
        assert_same(to_np(send), sc, "send")
        assert_same(to_np(R), Rc, "residual")
        recv = torch.from_numpy(rng.choice(specials, (N, stride)).astype(np.float32)).to(DEV)
        out = torch.zeros(D, device=DEV)
        oc = np.zeros(D, np.float32)
        B.covap_decompress(plan, t, recv, out)
        oracle.decompress(tab, K, t, to_np(recv), oc)
        assert_same(to_np(out), oc, "dense")


def test_k1_identity_on_gpu(B):
    wl = workloads.config(1)
    plan, tab = make_plans(B, wl.numel, wl.shard_elems, 1)
    G = workloads.gradient(wl, 0, 0, DEV)
    R = torch.zeros_like(G)
    send = torch.zeros_like(G)
    B.covap_compress(plan, 5, G, R, send)
    torch.cuda.synchronize()
    assert torch.equal(send, G) and not R.any()


def test_argument_errors(B):
    plan, _ = make_plans(B, [10_000], 1024, 4)
    G = torch.zeros(10_000, device=DEV)
    R = torch.zeros(10_000, device=DEV)
    send = torch.zeros(plan.packed_elems_max, device=DEV)
    with pytest.raises(B.CovapError) as e:
        B.covap_compress(plan, 0, G, R, send, send_cap_elems=10)
    assert e.value.status == 1
    with pytest.raises(B.CovapError):
        B.covap_compress(plan, 0, torch.zeros(10_001, device=DEV)[1:], R, send)   # misaligned
    # the binding refuses buffers that are too small or of the wrong element width before any address is taken
    with pytest.raises(ValueError):
        B.covap_compress(plan, 0, G[:9_999], R, send)
    with pytest.raises(ValueError):
        B.covap_compress(plan, 0, G, R.to(torch.bfloat16), send)
    with pytest.raises(ValueError):
        B.covap_compress(plan, 0, G, R, send, send_cap_elems=send.numel() + 1)
    with pytest.raises(ValueError):
        B.covap_decompress(plan, 0, send, G[:9_000], n_workers=1, stride_elems=send.numel())
    with pytest.raises(ValueError):
        B.covap_decompress(plan, 0, send, G, n_workers=2, stride_elems=send.numel())     # second row missing
    mplan = B.covap_plan([1000, 1000], 0, 2, bucket_cap_bytes=4, mode=B.COVAP_SHARD_MEDIAN)
    assert mplan.total_elems == 2024                            # 1 KiB padding after the first tensor
    with pytest.raises(ValueError):
        B.covap_compress(mplan, 0, torch.zeros(2000, device=DEV), torch.zeros(2024, device=DEV),
                         torch.zeros(1024, device=DEV))
    with pytest.raises(B.CovapError):
        B.covap_compress(plan, 0, G, G, send)                   # overlap
    with pytest.raises(B.CovapError) as e:
        B.covap_compress(plan, 0, G, R, send, bucket=99)
    assert e.value.status == 4
    with pytest.raises(B.CovapError):
        B.covap_decompress(plan, 0, send, G, n_workers=0, stride_elems=send.numel())
    with pytest.raises(B.CovapError):
        B.covap_decompress(plan, 0, torch.zeros(2 * send.numel(), device=DEV), G, n_workers=2,
                           stride_elems=send.numel() // 2 - 1)       # rows shorter than the payload
    torch.cuda.synchronize()


# ------------------------------------------------------------------ median sharding (Sec. III-C)

MEDIAN_CASES = [
    # layers, K, cap_bytes, ref
    ([41_011, 167_813, 1_074_805, 70_794, 76_697, 5_551], 4, 4, 55_903),      # Table V / 100, one layer per tensor
    ([41_011, 167_813, 1_074_805, 70_794, 76_697, 5_551], 8, 4, 0),
    ([1_003, 2_001, 30_007, 5, 4_099, 17, 90_001, 3], 3, 20_000, 0),           # ragged everywhere
    ([257] * 300, 5, 4, 0),                                                    # more shards than one launch carries
    ([100_000, 7], 16, 1 << 20, 1_000),                                        # capped at K pieces
    ([3_000_000, 5], 2, 25 << 20, 0),                                          # a shard of ~12 k tiles beside a tiny one
    ([2_500_000, 7], 2, 4, 0),                                                 # the same, one layer per tensor
    ([9_000_000, 300, 2_000_000, 11], 3, 4, 1_000_000),                        # pieces of ~3 M elements
]


@pytest.mark.parametrize("layers,K,cap,ref", MEDIAN_CASES)
def test_median_sharded_plans(B, layers, K, cap, ref):
    wl = workloads.scaled_down(workloads.config(3), layers, 4096)
    plans = make_median_plans(B, layers, K, cap_bytes=cap, ref=ref)
    run_iterations(B, wl, layers, 0, K, 3, 2 * K + 1, c=0.5, plans=plans, slack=3)
    plans = make_median_plans(B, layers, K, cap_bytes=cap, ref=ref)
    run_iterations(B, wl, layers, 0, K, 2, K + 1, per_bucket=True, plans=plans)


def test_median_sharded_bf16_and_knobs(B):
    layers = [1_003, 2_001, 30_007, 5, 4_099, 17, 90_001, 3]
    wl = workloads.scaled_down(workloads.config(3), layers, 4096)
    old = {k: B.covap_tune_get(k) for k in KNOBS}
    try:
        for k in KNOBS:
            B.covap_tune_set(k, KNOBS[k][-1])
        for dtype in (torch.float32, torch.bfloat16):
            plans = make_median_plans(B, layers, 4, dtype=dtype, cap_bytes=40_000)
            run_iterations(B, wl, layers, 0, 4, 5, 6, dtype=dtype, plans=plans)
    finally:
        for k in old:
            B.covap_tune_set(k, -1)                    # back to never set
    plans = make_median_plans(B, layers, 4, dtype=torch.bfloat16, cap_bytes=40_000)
    run_iterations(B, wl, layers, 0, 4, 3, 9, dtype=torch.bfloat16, plans=plans, c=0.25)


def test_median_sharded_long_shards_bf16_and_largest_launch_shapes(B):
    """Shards of millions of elements with the largest tiles (8192 elements) and in bf16, whole-arena and
    bucket by bucket: sent and unsent tiles are dealt out in alternating blocks inside one launch."""
    layers = [2_500_000, 7, 1_300_001]
    wl = workloads.scaled_down(workloads.config(3), layers, 4096)
    old = {k: B.covap_tune_get(k) for k in KNOBS}
    try:
        for k in KNOBS:
            B.covap_tune_set(k, KNOBS[k][-1])
        for dtype in (torch.float32, torch.bfloat16):
            plans = make_median_plans(B, layers, 2, dtype=dtype, cap_bytes=4)
            run_iterations(B, wl, layers, 0, 2, 3, 3, dtype=dtype, plans=plans)
            plans = make_median_plans(B, layers, 2, dtype=dtype, cap_bytes=4)
            run_iterations(B, wl, layers, 0, 2, 2, 3, dtype=dtype, plans=plans, per_bucket=True, c=0.5)
    finally:
        for k in old:
            B.covap_tune_set(k, -1)                    # back to never set
    for dtype in (torch.float32, torch.bfloat16):
        plans = make_median_plans(B, layers, 3, dtype=dtype, cap_bytes=25 << 20, ref=400_000)
        run_iterations(B, wl, layers, 0, 3, 2, 7, dtype=dtype, plans=plans)


# ------------------------------------------------------------------ HIP graph capture

def test_per_bucket_calls_under_hip_graph_replay(B):
    """Per-bucket launches captured once per residue of the step and replayed: every
    replay, with eager work and synchronisations in between, must give the bits the
    oracle gives for that step (the launches use no memset nodes and no allocation)."""
    numel, S, K, N = [300_000, 12_345], 8192, 3, 4
    wl = workloads.scaled_down(workloads.config(2), numel, S)
    plan, tab = make_plans(B, numel, S, K, cap_bytes=100_000)
    D = tab.D
    stride = (plan.packed_elems_max + 3) // 4 * 4
    G = torch.empty(D, device=DEV)
    R = torch.zeros(D, device=DEV)
    recv = torch.zeros(N, stride, device=DEV)
    out = torch.zeros(D, device=DEV)
    side = torch.cuda.Stream()
    graphs = []
    for r in range(K):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for b in range(tab.n_buckets):
                B.covap_compress(plan, r, G, R, recv[0], ef_coeff=0.5, bucket=b)
            for b in range(tab.n_buckets):
                B.covap_decompress(plan, r, recv, out, bucket=b)
        graphs.append(g)
    R.zero_()
    Rc = np.zeros(D, np.float32)
    for t in range(3 * K + 1):
        G.copy_(workloads.gradient(wl, 0, t, DEV))
        recv.copy_(workloads.payload_rows(wl, N, stride, t, DEV, first_worker=0))
        recv_c = to_np(recv)
        torch.cuda.synchronize()
        graphs[t % K].replay()
        scratch = torch.randn(1000, device=DEV).sum().item()       # eager work between replays
        torch.cuda.synchronize()
        oracle.compress(tab, K, t, to_np(G), Rc, recv_c[0], 0.5)
        out_c = np.zeros(D, np.float32)
        oracle.decompress(tab, K, t, recv_c, out_c)
        assert_same(to_np(recv[0]), recv_c[0], f"send t={t}")
        assert_same(to_np(R), Rc, f"residual t={t}")
        assert_same(to_np(out), out_c, f"dense t={t}")
        assert scratch == scratch


def test_per_bucket_calls_on_three_streams_inside_a_hip_graph(B):
    """The per-bucket launches dealt out to three streams inside the capture (bucket b on stream b mod 3, a
    bucket's decompress after its compress on the same stream; fork and join events become graph edges).  Buckets
    touch disjoint ranges, so any interleaving must give the oracle's bits, replay after replay."""
    numel, S, K, N = [300_000, 12_345, 200_001], 8192, 3, 4
    wl = workloads.scaled_down(workloads.config(2), numel, S)
    plan, tab = make_plans(B, numel, S, K, cap_bytes=100_000)
    D = tab.D
    stride = (plan.packed_elems_max + 3) // 4 * 4
    G = torch.empty(D, device=DEV)
    R = torch.zeros(D, device=DEV)
    recv = torch.zeros(N, stride, device=DEV)
    out = torch.zeros(D, device=DEV)
    main, sides = torch.cuda.Stream(), [torch.cuda.Stream() for _ in range(3)]
    graphs = []
    for r in range(K):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=main):
            fork = torch.cuda.Event()
            fork.record(main)
            for st in sides:
                st.wait_event(fork)
            for b in range(tab.n_buckets):
                B.covap_compress(plan, r, G, R, recv[0], ef_coeff=0.5, bucket=b, stream=sides[b % 3])
            for b in range(tab.n_buckets):
                B.covap_decompress(plan, r, recv, out, bucket=b, stream=sides[b % 3])
            for st in sides:
                join = torch.cuda.Event()
                join.record(st)
                main.wait_event(join)
        graphs.append(g)
    R.zero_()
    Rc = np.zeros(D, np.float32)
    for t in range(2 * K + 1):
        G.copy_(workloads.gradient(wl, 0, t, DEV))
        recv.copy_(workloads.payload_rows(wl, N, stride, t, DEV, first_worker=0))
        recv_c = to_np(recv)
        torch.cuda.synchronize()
        graphs[t % K].replay()
        scratch = torch.randn(1000, device=DEV).sum().item()       # eager work between replays
        torch.cuda.synchronize()
        oracle.compress(tab, K, t, to_np(G), Rc, recv_c[0], 0.5)
        out_c = np.zeros(D, np.float32)
        oracle.decompress(tab, K, t, recv_c, out_c)
        assert_same(to_np(recv[0]), recv_c[0], f"send t={t}")
        assert_same(to_np(R), Rc, f"residual t={t}")
        assert_same(to_np(out), out_c, f"dense t={t}")
        assert scratch == scratch


# ------------------------------------------------------------------ bf16 gradients, fp32 residual

@pytest.mark.parametrize("numel,S,K,c", [([100_003], 4096, 3, 1.0), ([7], 8, 2, 0.5), ([8 * 4096 + 9], 8192, 4, 0.3),
                                         ([768 * 768, 3072 * 768 + 5], 1 << 18, 6, 1.0)])
def test_mixed_precision_bf16_with_fp32_residual(B, numel, S, K, c):
    wl = workloads.scaled_down(workloads.config(4), numel, S)
    plan = B.covap_plan(numel, S, K, dtype=B.COVAP_BF16_RES32)
    tab = oracle.plan_fixed(numel, S, (25 << 20) // 2)
    D, N = tab.D, 3
    stride = (plan.packed_elems_max + 7) // 8 * 8
    R = torch.zeros(D, dtype=torch.float32, device=DEV)
    Rc = np.zeros(D, np.float32)
    old = {k: B.covap_tune_get(k) for k in ("compress_threads", "compress_unroll", "nontemporal")}
    try:
        for t in range(2 * K + 1):
            B.covap_tune_set("compress_threads", (64, 256)[t % 2])
            B.covap_tune_set("compress_unroll", (1, 2, 4)[t % 3])
            B.covap_tune_set("nontemporal", (t // 2) % 2)
            G = workloads.gradient(wl, 0, t, DEV, torch.bfloat16)
            recv = torch.full((N, stride), float("nan"), dtype=torch.bfloat16, device=DEV)
            recv_c = to_np(recv)
            B.covap_compress(plan, t, G, R, recv[0], ef_coeff=c)
            oracle.compress(tab, K, t, to_np(G), Rc, recv_c[0], c)
            torch.cuda.synchronize()
            assert_same(to_np(recv[0]), recv_c[0], f"send t={t}")
            assert_same(to_np(R), Rc, f"residual t={t}")
            recv[1:] = workloads.payload_rows(wl, N - 1, stride, t, DEV, torch.bfloat16)
            own_row = recv_c[0].copy()                   # the oracle averages its own payload, not the GPU's
            recv_c = to_np(recv)
            recv_c[0] = own_row
            out = torch.zeros(D, dtype=torch.bfloat16, device=DEV)
            out_c = np.zeros(D, np.uint16)
            B.covap_decompress(plan, t, recv, out)
            oracle.decompress(tab, K, t, recv_c, out_c)
            torch.cuda.synchronize()
            assert_same(to_np(out), out_c, f"dense t={t}")
    finally:
        for k in old:
            B.covap_tune_set(k, -1)                    # back to never set


def test_mixed_precision_on_median_shards(B):
    layers = [1_003, 2_001, 30_007, 5, 4_099, 17, 90_001, 3]
    wl = workloads.scaled_down(workloads.config(3), layers, 4096)
    K = 4
    plan = B.covap_plan(layers, 0, K, dtype=B.COVAP_BF16_RES32, bucket_cap_bytes=40_000,
                        mode=B.COVAP_SHARD_MEDIAN)
    tab = oracle.plan_median(layers, 20_000, K, 0, 512)         # 1 KiB of bf16
    D = tab.D
    assert plan.total_elems == D
    R = torch.zeros(D, device=DEV)
    Rc = np.zeros(D, np.float32)
    stride = (plan.packed_elems_max + 7) // 8 * 8
    for t in range(2 * K + 1):
        G = workloads.gradient(wl, 0, t, DEV, torch.bfloat16)
        G = torch.cat([G, torch.ones(D - G.numel(), dtype=torch.bfloat16, device=DEV)])
        send = torch.full((stride,), float("nan"), dtype=torch.bfloat16, device=DEV)
        sc = to_np(send)
        B.covap_compress(plan, t, G, R, send, ef_coeff=0.5)
        oracle.compress(tab, K, t, to_np(G), Rc, sc, 0.5)
        torch.cuda.synchronize()
        assert_same(to_np(send), sc, f"send t={t}")
        assert_same(to_np(R), Rc, f"residual t={t}")


def test_scheduler_driven_run(B):
    """A whole schedule of the error-feedback scheduler (Sec. III-D): the
    coefficient comes from covap_ef_coeff on one side and the oracle's formula on
    the other, step by step, while it climbs from 0.25 to 1."""
    numel, S, K, N = [150_001], 4096, 4, 2
    wl = workloads.scaled_down(workloads.config(1), numel, S)
    plan, tab = make_plans(B, numel, S, K)
    D = tab.D
    stride = (plan.packed_elems_max + 3) // 4 * 4
    R = torch.zeros(D, device=DEV)
    Rc = np.zeros(D, np.float32)
    seen = set()
    for t in range(26):
        c = B.covap_ef_coeff(0.25, t, 3, 0.125)
        cc = oracle.ef_coeff(0.25, t, 3, 0.125)
        assert np.float32(c) == np.float32(cc)
        seen.add(c)
        G = workloads.gradient(wl, 0, t, DEV)
        send = torch.zeros(stride, device=DEV)
        sc = np.zeros(stride, np.float32)
        B.covap_compress(plan, t, G, R, send, ef_coeff=c)
        oracle.compress(tab, K, t, to_np(G), Rc, sc, cc)
        torch.cuda.synchronize()
        assert_same(to_np(send), sc, f"send t={t}")
        assert_same(to_np(R), Rc, f"residual t={t}")
    assert min(seen) == 0.25 and max(seen) == 1.0 and len(seen) == 7


# ------------------------------------------------------------------ aliased residual

@pytest.mark.parametrize("mode,numel,S,K,dtype", [
    ("fixed", [100_003], 4096, 3, torch.float32), ("fixed", [7], 4, 2, torch.float32),
    ("fixed", [8 * 4096 + 9], 8192, 4, torch.bfloat16), ("fixed", [300_000, 12_345], 8192, 16, torch.float32),
    ("median", [1_003, 2_001, 30_007, 5, 4_099, 17, 90_001, 3], 0, 3, torch.float32),
    ("median", [257] * 300, 0, 5, torch.bfloat16),
])
def test_aliased_residual_compress(B, mode, numel, S, K, dtype):
    """covap_compress_aliased against the oracle, and against covap_compress itself
    (c = 1) when the accumulation buffer is fed the way a producer would."""
    wl = workloads.scaled_down(workloads.config(1), numel, 4096)
    if mode == "fixed":
        plan, tab = make_plans(B, numel, S, K, dtype, cap_bytes=60_000)
    else:
        plan, tab = make_median_plans(B, numel, K, dtype, cap_bytes=20_000)
    D = tab.D
    epv = 4 if dtype == torch.float32 else 8
    stride = (plan.packed_elems_max + epv - 1) // epv * epv
    acc = torch.zeros(D, dtype=dtype, device=DEV)
    acc_c = to_np(acc)
    R = torch.zeros(D, dtype=dtype, device=DEV)
    covered = np.zeros(D, bool)                                  # arena padding belongs to no shard
    for s_ in range(tab.n_shards):
        covered[int(tab.off[s_]):int(tab.off[s_] + tab.len[s_])] = True
    covered_t = torch.from_numpy(covered).to(DEV)
    for t in range(2 * K + 1):
        G = workloads.gradient(wl, 0, t, DEV, dtype)
        if G.numel() < D:
            G = torch.cat([G, torch.zeros(D - G.numel(), dtype=dtype, device=DEV)])
        G = G * covered_t
        acc = (G.float() + acc.float()).to(dtype)               # the producer accumulates
        acc_c = to_np(acc)
        send_a = torch.full((stride,), float("nan"), dtype=dtype, device=DEV)
        send_c = to_np(send_a)
        send_r = torch.full((stride,), float("nan"), dtype=dtype, device=DEV)
        per_bucket = t % 2 == 1
        for b in (range(tab.n_buckets) if per_bucket else [-1]):
            B.covap_compress_aliased(plan, t, acc, send_a, bucket=b)
            oracle.compress_aliased(tab, K, t, acc_c, send_c, bucket=b)
        B.covap_compress(plan, t, G, R, send_r)
        torch.cuda.synchronize()
        assert_same(to_np(send_a), send_c, f"send t={t}")
        assert_same(to_np(acc), acc_c, f"accum t={t}")
        assert_same(to_np(send_a), to_np(send_r), f"aliased vs plain payload t={t}")
        assert_same(to_np(acc), to_np(R), f"aliased buffer vs plain residual t={t}")


def test_aliased_rejects_mixed_precision(B):
    plan = B.covap_plan([1000], 64, 2, dtype=B.COVAP_BF16_RES32)
    a = torch.zeros(1000, dtype=torch.bfloat16, device=DEV)
    s = torch.zeros(1000, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.CovapError) as e:
        B.covap_compress_aliased(plan, 0, a, s)
    assert e.value.status == 5


# ------------------------------------------------------------------ more corners

@pytest.mark.parametrize("numel,S,K,N", [
    ([50_001], 4096, 1000, 2),          # interval far larger than the shard count
    ([50_001], 4096, (1 << 31) - 1, 2), # the largest interval the ratio policy hands out
    ([50_001], 4096, 13, 130),          # many workers, not a power of two
    ([4096 * 40], 4096, 40, 1),         # exactly one shard per step, single worker
    ([123_457], 4, 3, 2),               # smallest legal shard: tens of thousands of shards
])
def test_extreme_intervals_and_worker_counts(B, numel, S, K, N):
    wl = workloads.scaled_down(workloads.config(1), numel, S)
    plan, tab = make_plans(B, numel, S, K)
    D = tab.D
    stride = (plan.packed_elems_max + 64 + 3) // 4 * 4        # stride larger than the payload
    R = torch.zeros(D, device=DEV)
    Rc = np.zeros(D, np.float32)
    for t in [0, 1, K - 1, K, 10 ** 15 + 3]:
        G = workloads.gradient(wl, 0, t % 1000, DEV)
        recv = workloads.payload_rows(wl, N, stride, t % 1000, DEV, first_worker=0)
        recv_c = to_np(recv)
        B.covap_compress(plan, t, G, R, recv[0], ef_coeff=0.5)
        oracle.compress(tab, K, t, to_np(G), Rc, recv_c[0], 0.5)
        out = torch.full((D,), float("nan"), device=DEV)
        out_c = np.zeros(D, np.float32)
        B.covap_decompress(plan, t, recv, out, n_workers=N, stride_elems=stride)
        oracle.decompress(tab, K, t, recv_c, out_c)
        torch.cuda.synchronize()
        assert_same(to_np(recv[0]), recv_c[0], f"send t={t}")
        assert_same(to_np(R), Rc, f"residual t={t}")
        assert_same(to_np(out), out_c, f"dense t={t}")


def test_two_streams_run_independent_plans(B):
    """Two plans driven from two HIP streams at once give the results each gives alone
    (the library keeps no state between calls besides the immutable plans)."""
    cases = [([200_003], 4096, 3), ([150_001, 77], 8192, 5)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    state = []
    for (numel, S, K), st in zip(cases, streams):
        wl = workloads.scaled_down(workloads.config(1), numel, S)
        plan, tab = make_plans(B, numel, S, K)
        D = tab.D
        stride = (plan.packed_elems_max + 3) // 4 * 4
        state.append(dict(wl=wl, plan=plan, tab=tab, K=K, D=D, stride=stride,
                          R=torch.zeros(D, device=DEV), Rc=np.zeros(D, np.float32)))
    torch.cuda.synchronize()
    for t in range(6):
        pending = []
        for s_, st in zip(state, streams):
            G = workloads.gradient(s_["wl"], 0, t, DEV)
            send = torch.zeros(s_["stride"], device=DEV)
            torch.cuda.synchronize()
            B.covap_compress(s_["plan"], t, G, s_["R"], send, stream=st)
            pending.append((s_, G, send))
        torch.cuda.synchronize()
        for s_, G, send in pending:
            sc = np.zeros(s_["stride"], np.float32)
            oracle.compress(s_["tab"], s_["K"], t, to_np(G), s_["Rc"], sc)
            assert_same(to_np(send), sc, f"send t={t}")
            assert_same(to_np(s_["R"]), s_["Rc"], f"residual t={t}")


# ------------------------------------------------------------------ seeded random shapes

@pytest.mark.parametrize("seed", range(12))
def test_random_layouts_intervals_and_worker_counts(B, seed):
    """Seeded random cases: tensor lists, shard sizes, intervals, worker counts, element
    types, both sharding modes and per-bucket calls, a few iterations each, every output
    against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    n_t = int(rng.integers(1, 7))
    numel = [int(x) for x in rng.integers(1, 60_000, n_t)]
    dtype = (torch.float32, torch.bfloat16)[int(rng.integers(0, 2))]
    epv = 4 if dtype == torch.float32 else 8
    K = int(rng.integers(1, 9))
    N = int(rng.integers(1, 6))
    c = float(rng.choice([1.0, 0.5, 0.3]))
    per_bucket = bool(rng.integers(0, 2))
    if rng.integers(0, 2):
        S = int(rng.choice([1, 2, 8, 31, 256, 1000])) * epv
        cap = int(rng.choice([S * epv, 40_000, 25 << 20]))
        wl = workloads.scaled_down(workloads.config(2), numel, S)
        run_iterations(B, wl, numel, S, K, N, K + 2, dtype=dtype, c=c, per_bucket=per_bucket, cap_bytes=cap)
    else:
        cap = int(rng.choice([4, 20_000, 200_000]))
        wl = workloads.scaled_down(workloads.config(3), numel, 4096)
        plans = make_median_plans(B, numel, K, dtype=dtype, cap_bytes=cap)
        run_iterations(B, wl, numel, 0, K, N, K + 2, dtype=dtype, c=c, per_bucket=per_bucket, plans=plans)


def test_bf16_rounding_over_the_float32_pattern_space(B):
    """Every upper half (sign, exponent, top mantissa bits: 65,536 values) crossed with 64
    lower halves (ties, their neighbours, extremes, random): 4.2 M fp32 patterns, incl.
    subnormals, Inf and NaN, pushed through the kernel's fp32 -> bf16 rounding (the
    fp32-residual mode with G = 0, c = 1 sends bf16(R)) and compared with the oracle."""
    rng = np.random.default_rng(9)
    lows = np.unique(np.r_[[0x0000, 0x0001, 0x7fff, 0x8000, 0x8001, 0xffff, 0x4000, 0xc000],
                           rng.integers(0, 1 << 16, 56)]).astype(np.uint32)
    pats = ((np.arange(1 << 16, dtype=np.uint32)[:, None] << 16) | lows[None, :]).ravel()
    n = pats.size // 8 * 8
    pats = pats[:n]
    Rn = pats.view(np.float32).copy()
    S = 1 << 16
    plan = B.covap_plan([n], S, 1, dtype=B.COVAP_BF16_RES32)
    tab = oracle.plan_fixed([n], S, 1 << 40)
    G = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    R = torch.from_numpy(Rn).to(DEV)
    send = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    B.covap_compress(plan, 0, G, R, send)
    torch.cuda.synchronize()
    Rc = Rn.copy()
    sc = np.zeros(n, np.uint16)
    oracle.compress(tab, 1, 0, np.zeros(n, np.uint16), Rc, sc)
    got = to_np(send)
    nan = np.isnan(Rn)
    assert np.array_equal(got[~nan], sc[~nan])                       # every finite and infinite pattern, bit for bit
    assert np.all((got[nan] & 0x7f80) == 0x7f80) and np.all((got[nan] & 0x007f) != 0)   # NaN stays NaN
    assert_same(to_np(R)[~nan], Rc[~nan], "residual")


def test_empty_arena_is_a_no_op(B):
    """No elements: every hot-path call succeeds, launches nothing and leaves the buffers alone."""
    for mode in (B.COVAP_SHARD_FIXED, B.COVAP_SHARD_MEDIAN):
        plan = B.covap_plan([0, 0], 8, 2, mode=mode)
        G = torch.full((16,), 3.0, device=DEV)
        R = torch.full((16,), 4.0, device=DEV)
        send = torch.full((16,), 5.0, device=DEV)
        recv = torch.full((2, 16), 6.0, device=DEV)
        out = torch.full((16,), 7.0, device=DEV)
        for t in range(3):
            B.covap_compress(plan, t, G, R, send)
            B.covap_compress_aliased(plan, t, R, send)
            B.covap_decompress(plan, t, recv, out)
        torch.cuda.synchronize()
        assert bool((R == 4.0).all()) and bool((send == 5.0).all()) and bool((out == 7.0).all())
    ws = torch.empty(max(B.topk_workspace_bytes(0), 256), dtype=torch.uint8, device=DEV)
    B.topk_compress(G, R, 0, send, recv.view(torch.int32)[0], ws, n=0)       # n = 0: nothing to do
    torch.cuda.synchronize()
    assert bool((R == 4.0).all())


def test_long_run_conserves_every_gradient_on_the_device(B):
    """100 iterations on integer-valued gradients (sums stay exact in fp32), c = 1: at the
    end, everything that was ever sent plus the residual equals the sum of all gradients,
    element by element and exactly -- the telescoped form of Algorithm 1's invariant, checked
    on the GPU path over a run as long as the benchmark configurations ask for.  The oracle
    runs the same 100 iterations on its own residual; payload and residual are compared with
    it every tenth iteration and at the end."""
    numel, S, K, T = [300_007, 65_536, 11], 8192, 5, 100
    plan, tab = make_plans(B, numel, S, K)
    D = tab.D
    stride = (plan.packed_elems_max + 3) // 4 * 4
    R = torch.zeros(D, device=DEV)
    Rc = np.zeros(D, np.float32)
    total_grad = torch.zeros(D, dtype=torch.float64, device=DEV)
    total_sent = torch.zeros(D, dtype=torch.float64, device=DEV)
    send = torch.zeros(stride, device=DEV)
    for t in range(T):
        G = workloads.integer_valued(D, seed=900 + t, lo=-500, hi=500, device=DEV)
        total_grad += G
        send.fill_(float("nan"))
        B.covap_compress(plan, t, G, R, send)
        sc = np.full(stride, np.nan, np.float32)
        oracle.compress(tab, K, t, G.cpu().numpy(), Rc, sc)
        p = 0
        for s in plan.selected(t):                       # independent unpack from the plan's shard list
            off, ln, _ = plan.shard(s)
            total_sent[off:off + ln] += send[p:p + ln]
            p += ln
        assert p == plan.packed_elems(t)
        if t % 10 == 0 or t == T - 1:
            torch.cuda.synchronize()
            assert_same(to_np(send), sc, f"send t={t}")
            assert_same(to_np(R), Rc, f"residual t={t}")
    torch.cuda.synchronize()
    assert torch.equal(total_sent + R.double(), total_grad)
    assert int((R != 0).sum()) > 0
