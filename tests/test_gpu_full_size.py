"""GPU parity at the benchmark configurations' real sizes, for as many iterations as
the measurement plan fixes: every iteration of the ResNet-50-shaped run, the first
2K+1 of the VGG-19-, BERT-base- and GPT-2-medium-shaped runs (every shard is sent
twice, so accumulate -> send -> clear -> accumulate happens at full size), in the
benchmark's launch configuration (payload mode, default knobs, its row stride).
Every element of the payload, the residual and the dense result is compared with the
oracle after every step, and so is the dense result of the form that takes one summed
payload row (the step after a sum-AllReduce).  The same sets under the paper's own sharding (Sec. III-C:
25 MiB communication tensors cut by the median rule into pieces of several million
elements), whole-arena and bucket by bucket.

The oracle's C routines are called on runs of whole shards from a thread pool here
(same routines, same per-element order), which keeps these runs to seconds per step.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2311_04499_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
THREADS = max(1, min(16, os.cpu_count() or 1))


@pytest.fixture(scope="module")
def B():
    from paper_2311_04499_amd import binding
    binding.lib()
    assert torch.cuda.is_available()
    return binding


def to_np(t):
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def as_int(t):
    return t.view(torch.int32 if t.element_size() == 4 else torch.int16)


def same_bits(gpu, cpu, what):
    """gpu: device tensor; cpu: the oracle's array.  Compared on the device (the oracle's
    array goes up once); on a mismatch, say where."""
    want = torch.from_numpy(cpu.view(np.int32 if cpu.itemsize == 4 else np.int16)).to(DEV)
    got = as_int(gpu)
    if torch.equal(got, want):
        return
    bad = torch.nonzero(got != want).flatten()
    i = int(bad[0])
    raise AssertionError(f"{what}: {bad.numel()} of {got.numel()} elements differ, first at {i}: "
                         f"got bits {int(got[i])} want {int(want[i])}")


KINDS = {  # element type of (gradient and dense result, residual, payload) and the plan's code
    "f32": (torch.float32, torch.float32, torch.float32, "COVAP_F32"),
    "bf16": (torch.bfloat16, torch.bfloat16, torch.bfloat16, "COVAP_BF16"),
    "bf16_res32": (torch.bfloat16, torch.float32, torch.bfloat16, "COVAP_BF16_RES32"),
    "f32_pay16": (torch.float32, torch.float32, torch.float16, "COVAP_F32_PAY16"),
}


def np_of(dtype):
    return np.float32 if dtype == torch.float32 else np.uint16


def run_payload_mode(B, wl, plan, tab, steps, kind="f32", per_bucket=lambda t: False, c=1.0):
    """Worker 0 runs the real compress every step (its residual carries over); rows 1..N-1 of
    the receive buffer are synthetic payloads at packed shape, uploaded once; gradients cycle
    through a ring of three generated sets."""
    gdt, rdt, pdt, _ = KINDS[kind]
    K, N, D = wl.K, wl.n_workers, tab.D
    stride = (plan.packed_elems_max + 1023) // 1024 * 1024       # the benchmark's row stride
    recv = torch.empty(N, stride, dtype=pdt, device=DEV)
    recv[1:] = workloads.payload_rows(wl, N - 1, stride, 0, DEV, pdt)
    recv_c = to_np(recv)
    ring, ring_c = [], []
    for i in range(3):
        G = workloads.gradient(wl, 0, i, DEV, gdt)
        if G.numel() < D:                                        # alignment padding of variable-length shards
            G = torch.cat([G, torch.ones(D - G.numel(), dtype=gdt, device=DEV)])
        ring.append(G)
        ring_c.append(to_np(G))
    R = torch.zeros(D, dtype=rdt, device=DEV)
    Rc = np.zeros(D, np_of(rdt))
    out = torch.full((D,), float("nan"), dtype=gdt, device=DEV)
    out_c = to_np(out)
    nb = tab.n_buckets
    for t in steps:
        buckets = range(nb) if per_bucket(t) else [-1]
        recv[0].fill_(float("nan"))
        recv_c[0] = to_np(recv[0])
        for b in buckets:
            B.covap_compress(plan, t, ring[t % 3], R, recv[0], ef_coeff=c, bucket=b)
        for b in buckets:
            B.covap_decompress(plan, t, recv, out, n_workers=N, stride_elems=stride, bucket=b)
        assert plan.packed_elems(t) == oracle.packed_elems(tab, K, t)
        oracle.compress(tab, K, t, ring_c[t % 3], Rc, recv_c[0], c, threads=THREADS)
        oracle.decompress(tab, K, t, recv_c, out_c, threads=THREADS)      # row 0 is the oracle's own payload
        torch.cuda.synchronize()
        same_bits(recv[0], recv_c[0], f"send t={t}")              # untouched positions keep the NaN prefill on both sides
        same_bits(R, Rc, f"residual t={t}")
        same_bits(out, out_c, f"dense t={t}")
        # the same step after a sum-AllReduce: the rows added up (here one after the other, in the
        # payload's own type) and handed over as one row
        acc = recv[0].clone()
        for w in range(1, N):
            acc += recv[w]
        out.fill_(float("nan"))
        out_c[:] = to_np(out)
        for b in buckets:
            B.covap_decompress_reduced(plan, t, acc, out, N, bucket=b)
        oracle.unpack_mean(tab, K, t, to_np(acc), N, out_c, threads=THREADS)
        torch.cuda.synchronize()
        same_bits(out, out_c, f"dense after a summed exchange t={t}")
    return R


def fixed_plans(B, wl, kind):
    gdt, _, _, code = KINDS[kind]
    esz = 4 if gdt == torch.float32 else 2
    plan = B.covap_plan(wl.numel, wl.shard_elems, wl.K, dtype=getattr(B, code))
    tab = oracle.plan_fixed(wl.numel, wl.shard_elems, (25 << 20) // esz)
    assert plan.total_elems == tab.D == wl.D and plan.num_shards == tab.n_shards
    return plan, tab


def median_plans(B, wl, kind):
    gdt, _, _, code = KINDS[kind]
    esz = 4 if gdt == torch.float32 else 2
    plan = B.covap_plan(wl.numel, 0, wl.K, dtype=getattr(B, code), mode=B.COVAP_SHARD_MEDIAN)
    tab = oracle.plan_median(wl.numel, (25 << 20) // esz, wl.K, 0, 1024 // esz)
    assert plan.total_elems == tab.D and plan.num_shards == tab.n_shards and plan.num_buckets == tab.n_buckets
    return plan, tab


def test_resnet50_shaped_run_every_iteration(B):
    wl = workloads.config(2)
    plan, tab = fixed_plans(B, wl, "f32")
    R = run_payload_mode(B, wl, plan, tab, range(wl.iterations))
    assert wl.iterations == 50 and bool((R != 0).any())


@pytest.mark.parametrize("cfg,dtype", [(3, "f32"), (4, "f32"), (4, "bf16"), (5, "f32"), (5, "bf16_res32"),
                                       (5, "f32_pay16")])
def test_first_two_periods_plus_one_at_full_size(B, cfg, dtype):
    wl = workloads.config(cfg)
    if cfg == 4:
        assert B.covap_ratio_from_ccr(6.0) == wl.K                # BERT's interval comes from CCR = 6
    plan, tab = fixed_plans(B, wl, dtype)
    last = tab.n_shards - 1
    steps = range(2 * wl.K + 1)
    assert any(plan.is_selected(t, last) == 1 for t in steps)    # the short last shard is sent on the way
    run_payload_mode(B, wl, plan, tab, steps, dtype)


@pytest.mark.parametrize("cfg,dtype", [(3, "f32"), (3, "bf16"), (5, "f32"), (5, "bf16")])
def test_paper_sharding_at_full_size(B, cfg, dtype):
    """Median sharding of the VGG-19- and GPT-2-medium-shaped sets: shards of millions of elements (thousands
    of tiles each, many dealing blocks).  First period whole-arena, second bucket by bucket, then one more
    step; the benchmark's --shard-mode median runs exactly these launches."""
    wl = workloads.config(cfg)
    plan, tab = median_plans(B, wl, dtype)
    assert int(tab.len.max()) > 4_000_000
    K = wl.K
    steps = range(2 * K + 1) if cfg == 3 else list(range(K)) + [K, K + 3, 2 * K - 1, 2 * K]
    run_payload_mode(B, wl, plan, tab, steps, dtype, per_bucket=lambda t: K <= t < 2 * K, c=0.5 if cfg == 3 else 1.0)
