#!/usr/bin/env python3
"""Benchmark of the COVAP hot path on one MI355X.

One "step" = one worker's whole per-iteration path on one synthetic gradient
set: covap_compress (error feedback + filter + pack + residual) followed by
covap_decompress (N-way mean + unpack + zero fill) over the N payload rows.
Inputs are resident in HBM before the timed region.  The default workload is
the GPT-2-medium-shaped gradient set (355M fp32 elements, shard 2^20, N = 64,
K = 16) in payload mode: row 0 of the receive buffer is this worker's own
packed output, rows 1..N-1 are synthetic payloads drawn at packed shape.

Prints ONE JSON line: metric / value (GB/s of gradient processed) / ms_per_step,
`roofline` for the slower of the two kernels (algorithmic HBM bytes over its
HIP-event duration, against the 8 TB/s peak), `kernels` (both), `cpu_baseline`
(the CPU oracle on one full iteration), and the contrast and streamed-mode
measurements.  `--gpus N` with N > 1 is refused: this build is a single-GPU
path with no collectives.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5")
    ap.add_argument("--dtype", choices=["f32", "bf16", "bf16_res32", "f32_pay16"], default="f32",
                    help="element type; bf16_res32 = bf16 gradients and payload, fp32 residual")
    ap.add_argument("--shard-mode", choices=["fixed", "median"], default="fixed",
                    help="fixed-size shards (default) or the median sharding of Sec. III-C")
    ap.add_argument("--tune", action="append", default=[], help="key=value launch knob")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-topk", action="store_true")
    ap.add_argument("--no-probes", action="store_true")
    ap.add_argument("--no-streamed", action="store_true",
                    help="skip the per-bucket / HIP-graph / overlap measurements")
    return ap.parse_args()


def read_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding across "
              "GPUs); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2311_04499_amd import binding as B
    from paper_2311_04499_amd import workloads

    B.lib()                                    # no fallback: fails if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    for kv in args.tune:
        k, v = kv.split("=")
        B.covap_tune_set(k, int(v))

    dev = "cuda:0"
    torch.cuda.set_device(0)
    wl = workloads.config(args.config)
    # gradient / dense result, residual, payload: element types and sizes
    tdtype = torch.float32 if args.dtype in ("f32", "f32_pay16") else torch.bfloat16
    rdtype = torch.bfloat16 if args.dtype == "bf16" else torch.float32
    pdtype = {"f32": torch.float32, "f32_pay16": torch.float16}.get(args.dtype, torch.bfloat16)
    esz = 4 if args.dtype in ("f32", "f32_pay16") else 2
    rsz = 2 if args.dtype == "bf16" else 4
    psz = 4 if args.dtype == "f32" else 2
    epv = 16 // psz
    plan = B.covap_plan(wl.numel, wl.shard_elems, wl.K,
                        dtype={"f32": B.COVAP_F32, "bf16": B.COVAP_BF16, "bf16_res32": B.COVAP_BF16_RES32,
                               "f32_pay16": B.COVAP_F32_PAY16}[args.dtype],
                        mode=B.COVAP_SHARD_FIXED if args.shard_mode == "fixed" else B.COVAP_SHARD_MEDIAN)
    D, N, K = plan.total_elems, wl.n_workers, wl.K
    P_max = plan.packed_elems_max
    stride = (P_max + 1023) // 1024 * 1024          # rows start on 2 KiB boundaries at least

    # ---- inputs, resident in HBM before anything is timed
    ring = [workloads.gradient(wl, 0, i, dev, tdtype) for i in range(3)]
    if D > wl.D:                               # median mode may pad bucket starts to 16 bytes
        ring = [torch.cat([g, g.new_zeros(D - wl.D)]) for g in ring]
    residual = torch.zeros(D, dtype=rdtype, device=dev)
    recv = torch.empty(N, stride, dtype=pdtype, device=dev)
    if N > 1:
        recv[1:] = workloads.payload_rows(wl, N - 1, stride, 0, dev, pdtype)
    dense = torch.empty(D, dtype=tdtype, device=dev)
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()

    def step(t):
        B.covap_compress(plan, t, ring[t % 3], residual, recv[0], stream=stream)
        B.covap_decompress(plan, t, recv, dense, n_workers=N, stride_elems=stride, stream=stream)

    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps, HIP events around every kernel
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t_first = args.warmup
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    for i in range(args.steps):
        t = t_first + i
        ev[i][0].record(stream)
        B.covap_compress(plan, t, ring[t % 3], residual, recv[0], stream=stream)
        ev[i][1].record(stream)
        B.covap_decompress(plan, t, recv, dense, n_workers=N, stride_elems=stride, stream=stream)
        ev[i][2].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0

    ms_step = wall * 1e3 / args.steps
    tc = [e[0].elapsed_time(e[1]) for e in ev]           # ms
    td = [e[1].elapsed_time(e[2]) for e in ev]
    tc_avg, td_avg = sum(tc) / len(tc), sum(td) / len(td)
    steps_t = [t_first + i for i in range(args.steps)]
    P_avg = sum(plan.packed_elems(t) for t in steps_t) / len(steps_t)
    bytes_c = esz * D + psz * P_avg + rsz * 2 * D        # read G, read R, write R, write packed
    bytes_d = psz * N * P_avg + esz * D                  # read N rows, write dense
    grad_gbs = esz * D / (ms_step * 1e-3) / 1e9
    hbm_gbs = (bytes_c + bytes_d) / (ms_step * 1e-3) / 1e9

    dominant = ("covap_decompress", td_avg, bytes_d) if td_avg >= tc_avg else \
               ("covap_compress", tc_avg, bytes_c)
    ach = dominant[2] / (dominant[1] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dominant[0], "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                # the committed counter summaries cover the default element type and sharding only
                "traffic": read_traffic(dominant[0], wl.name)
                if args.dtype == "f32" and args.shard_mode == "fixed" and not args.tune else None,
                "bytes_per_launch": round(dominant[2]), "avg_launch_us": round(dominant[1] * 1e3, 2)}

    def pct(xs, q):
        ys = sorted(xs)
        return round(ys[min(len(ys) - 1, int(q * len(ys)))] * 1e3, 2)

    kernels = {
        "covap_compress": {"avg_us": round(tc_avg * 1e3, 2), "p10_us": pct(tc, 0.1), "median_us": pct(tc, 0.5),
                           "p90_us": pct(tc, 0.9), "algorithmic_bytes": round(bytes_c),
                           "GB/s": round(bytes_c / (tc_avg * 1e-3) / 1e9, 1),
                           "frac": round(bytes_c / (tc_avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "covap_decompress": {"avg_us": round(td_avg * 1e3, 2), "p10_us": pct(td, 0.1), "median_us": pct(td, 0.5),
                             "p90_us": pct(td, 0.9), "algorithmic_bytes": round(bytes_d),
                             "GB/s": round(bytes_d / (td_avg * 1e-3) / 1e9, 1),
                             "frac": round(bytes_d / (td_avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
    }

    out = {
        "metric": "compress+decompress GB/s of gradient processed", "value": round(grad_gbs, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"cfg{wl.cfg_id}:{wl.name}", "elements": D, "shard_elems": wl.shard_elems,
                   "n_workers": N, "K": K, "mode": "payload", "sharding": args.shard_mode,
                   "shards": plan.num_shards},
        "hbm_GB/s": round(hbm_gbs, 1), "hbm_frac": round(hbm_gbs / HBM_PEAK_GBS, 4),
        "overhead_us_per_iter": round(ms_step * 1e3, 1),
        "roofline": roofline, "kernels": kernels,
    }

    # ---- achievable streaming rate in the same run (context for the fraction)
    if not args.no_probes:
        nb = min(D * esz, 1 << 31) // 16 * 16
        a = dense.view(torch.uint8)[:nb]
        b = ring[0].view(torch.uint8)[:nb]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            B.covap_probe_copy(a, b, nb, stream=stream)
        e0.record(stream)
        reps = 20
        for _ in range(reps):
            B.covap_probe_copy(a, b, nb, stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        copy_gbs = 2 * nb * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        out["probe_copy_GB/s"] = round(copy_gbs, 1)
        if args.dtype == "f32":
            # a = b + s*c: the two-reads-one-write shape of compress without its index work
            nt = nb // 4
            ta, tb, tc_ = dense[:nt], ring[0][:nt], ring[1][:nt]
            for _ in range(3):
                B.covap_probe_triad(ta, tb, tc_, 0.5, nt, stream=stream)
            e0.record(stream)
            for _ in range(reps):
                B.covap_probe_triad(ta, tb, tc_, 0.5, nt, stream=stream)
            e1.record(stream)
            torch.cuda.synchronize()
            out["probe_triad_GB/s"] = round(3 * nb * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)

    # ---- top-k contrast on the same gradient buffers
    if not args.no_topk and args.dtype == "f32":
        try:
            k = -(-D // 1000)                            # ceil(0.1% of D)
            ws_bytes = B.topk_workspace_bytes(D)
            ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
            vals = torch.empty(k, dtype=torch.float32, device=dev)
            idx = torch.empty(k, dtype=torch.int32, device=dev)
            res2 = torch.zeros(D, dtype=torch.float32, device=dev)
            for t in range(3):
                B.topk_compress(ring[t % 3], res2, k, vals, idx, ws, stream=stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = max(5, min(args.steps, 20))
            e0.record(stream)
            for t in range(reps):
                B.topk_compress(ring[t % 3], res2, k, vals, idx, ws, stream=stream)
            e1.record(stream)
            torch.cuda.synchronize()
            topk_us = e0.elapsed_time(e1) * 1e3 / reps
            out["topk"] = {"k": k, "us_per_iter": round(topk_us, 1),
                           "vs_covap_compress": round(topk_us / (tc_avg * 1e3), 2),
                           "vs_covap_compress_plus_decompress": round(topk_us / (ms_step * 1e3), 2)}
            del ws, vals, idx, res2
        except B.CovapError as e:
            out["topk"] = {"error": str(e)}

    # ---- Random-k (k = 1 %) and FP16 contrast kernels on the same gradient buffers
    if not args.no_topk and args.dtype == "f32":
        def timed_us(fn, reps=10):
            for t in range(2):
                fn(t)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for t in range(reps):
                fn(t)
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps

        try:
            res2 = torch.zeros(D, dtype=torch.float32, device=dev)
            k1 = -(-D // 100)
            g = torch.Generator(device=dev)
            g.manual_seed(workloads.seed_for(wl.cfg_id, 0, 0, stream=2))
            # distinct coordinates from a shared seed: one per stride-100 cell
            ridx = (torch.arange(k1, device=dev, dtype=torch.int64) * 100 +
                    torch.randint(0, 100, (k1,), generator=g, device=dev)).clamp_(max=D - 1)
            ridx = torch.unique(ridx).to(torch.int32)
            rvals = torch.empty(ridx.numel(), dtype=torch.float32, device=dev)
            us = timed_us(lambda t: B.randk_compress(ring[t % 3], res2, ridx, rvals, stream=stream))
            out["randk"] = {"k": int(ridx.numel()), "us_per_iter": round(us, 1),
                            "vs_covap_compress": round(us / (tc_avg * 1e3), 2)}
            half = torch.empty(D, dtype=torch.float16, device=dev)
            us = timed_us(lambda t: B.fp16_compress(ring[t % 3], res2, half, stream=stream))
            out["fp16"] = {"compress_us_per_iter": round(us, 1),
                           "vs_covap_compress": round(us / (tc_avg * 1e3), 2)}
            del half, res2, rvals, ridx
            if "topk" in out and "k" in out["topk"]:
                kk = out["topk"]["k"]
                sv = torch.randn(N, kk, device=dev)
                # N different ascending index rows: one coordinate per cell of D/kk elements
                cell = D // kk
                si = (torch.arange(kk, device=dev, dtype=torch.int64)[None, :] * cell +
                      torch.randint(0, cell, (N, kk), generator=g, device=dev)).to(torch.int32).contiguous()
                us = timed_us(lambda t: B.sparse_decompress_sorted(sv, si, dense, stream=stream), reps=5)
                us_pw = timed_us(lambda t: B.sparse_decompress(sv, si, dense, stream=stream), reps=3)
                out["topk"]["decompress_us_per_iter"] = round(us, 1)
                out["topk"]["decompress_per_worker_launches_us"] = round(us_pw, 1)
                out["topk"]["compress_plus_decompress_vs_covap"] = round(
                    (out["topk"]["us_per_iter"] + us) / (ms_step * 1e3), 2)
                del sv, si
        except B.CovapError as e:
            out["contrast_error"] = str(e)

    # ---- aliased-residual compress (the producer accumulates; never the headline number:
    # the error-feedback addition is then paid for inside the producer)
    if args.dtype not in ("bf16_res32", "f32_pay16"):
        acc_buf = ring[1].clone()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for t in range(K):
            B.covap_compress_aliased(plan, t, acc_buf, recv[0], stream=stream)
        e0.record(stream)
        for t in range(2 * K):
            B.covap_compress_aliased(plan, t, acc_buf, recv[0], stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (2 * K)
        P_period = sum(plan.packed_elems(t) for t in range(K)) / K
        out["aliased_compress"] = {"us_per_iter": round(us, 2), "algorithmic_bytes": round(3 * esz * P_period),
                                   "GB/s": round(3 * esz * P_period / (us * 1e-6) / 1e9, 1)}
        del acc_buf

    # ---- per-bucket streamed mode: one launch per communication bucket, as a DDP hook
    # would issue them while backward is still running (Sec. II-B); eager launches,
    # HIP graphs (one per residue of the step), and overlap with a synthetic backward
    if not args.no_streamed:
        nb = plan.num_buckets

        def per_bucket(t):
            for b in range(nb):
                B.covap_compress(plan, t, ring[0], residual, recv[0], bucket=b)
            for b in range(nb):
                B.covap_decompress(plan, t, recv, dense, n_workers=N, stride_elems=stride, bucket=b)

        def timed(fn, reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            w0 = time.perf_counter()
            e0.record()
            for t in range(reps):
                fn(t)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps, (time.perf_counter() - w0) * 1e6 / reps

        reps = max(K, min(args.steps, 2 * K))
        per_bucket(0)
        eager_gpu_us, eager_wall_us = timed(per_bucket, reps)
        sres = {"buckets": nb, "launches_per_step": 2 * nb,
                "eager_us_per_step": round(eager_wall_us, 1),
                "whole_arena_us_per_step": round(ms_step * 1e3, 1)}

        # what a bucket hook would do: compress bucket by bucket as the gradients become
        # ready, average everything in one call once the exchange is over
        def hook_like(t):
            for b in range(nb):
                B.covap_compress(plan, t, ring[0], residual, recv[0], bucket=b)
            B.covap_decompress(plan, t, recv, dense, n_workers=N, stride_elems=stride)

        hook_like(0)
        _, hook_wall_us = timed(hook_like, reps)
        sres["per_bucket_compress_one_decompress_us_per_step"] = round(hook_wall_us, 1)
        try:
            graphs = []
            side = torch.cuda.Stream()
            for r in range(K):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    per_bucket(r)
                graphs.append(g)
            for g in graphs:
                g.replay()
            _, graph_wall_us = timed(lambda t: graphs[t % K].replay(), reps)
            sres["graph_us_per_step"] = round(graph_wall_us, 1)
        except Exception as e:                              # reported, never hidden
            sres["graph_error"] = repr(e)[:200]

        # overlap: backward = one bf16 GEMM per bucket on the main stream; compress of
        # bucket b runs on a side stream as soon as "its gradient is ready"
        try:
            m = 4096
            xa = torch.randn(m, m, device=dev, dtype=torch.bfloat16)
            xb = torch.randn(m, m, device=dev, dtype=torch.bfloat16)
            xc = torch.empty(m, m, device=dev, dtype=torch.bfloat16)
            side = torch.cuda.Stream()
            ready = [torch.cuda.Event() for _ in range(nb)]
            done = torch.cuda.Event()

            def backward_only(t):
                for b in range(nb):
                    torch.mm(xa, xb, out=xc)

            def compress_only(t):
                for b in range(nb):
                    B.covap_compress(plan, t, ring[0], residual, recv[0], bucket=b)

            def overlapped(t):
                for b in range(nb):
                    torch.mm(xa, xb, out=xc)
                    ready[b].record()
                    side.wait_event(ready[b])
                    B.covap_compress(plan, t, ring[0], residual, recv[0], bucket=b, stream=side)
                done.record(side)
                torch.cuda.current_stream().wait_event(done)

            for f in (backward_only, compress_only, overlapped):
                f(0)
            bw_us, _ = timed(backward_only, reps)
            co_us, _ = timed(compress_only, reps)
            ov_us, _ = timed(overlapped, reps)
            sres["overlap"] = {"backward_us": round(bw_us, 1), "compress_us": round(co_us, 1),
                               "both_overlapped_us": round(ov_us, 1),
                               "exposed_compress_us": round(ov_us - bw_us, 1),
                               "hidden_frac": round(1.0 - max(ov_us - bw_us, 0.0) / co_us, 3)}
            del xa, xb, xc
        except Exception as e:
            sres["overlap_error"] = repr(e)[:200]
        out["streamed"] = sres

    # ---- CPU oracle on a bounded sample of the same workload (reported, not a target)
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        tab = oracle.plan_fixed(wl.numel, wl.shard_elems, (25 << 20) // esz) if args.shard_mode == "fixed" \
            else oracle.plan_median(wl.numel, (25 << 20) // esz, K, 0, 1024 // psz)
        t = t_first + args.steps
        to_np = lambda x: x.cpu().numpy() if x.dtype == torch.float32 else \
            x.cpu().view(torch.int16).numpy().view(np.uint16)
        # inputs are generated, never taken from the GPU path's outputs: a gradient, a residual
        # of the same scale, and the synthetic payload rows (row 0 is filled by the oracle itself)
        Gn = to_np(ring[t % 3])
        Rn = to_np(ring[(t + 1) % 3].to(rdtype)).copy()
        recv_n = to_np(recv).copy()
        recv_n[0] = 0
        out_n = np.empty(D, Gn.dtype)
        c0 = time.perf_counter()
        oracle.compress(tab, K, t, Gn, Rn, recv_n[0])
        c1 = time.perf_counter()
        oracle.decompress(tab, K, t, recv_n, out_n)
        c2 = time.perf_counter()
        out["cpu_baseline"] = {"value": round(esz * D / (c2 - c0) / 1e9, 4), "unit": "GB/s",
                               "cores": 1, "kind": "oracle",
                               "sample": "1 full iteration of the same workload (compress %.2f s + "
                                         "decompress %.2f s), single thread" % (c1 - c0, c2 - c1),
                               "compress_us_per_iter": round((c1 - c0) * 1e6),
                               "decompress_us_per_iter": round((c2 - c1) * 1e6),
                               "host_cpus": os.cpu_count(), "cpu_model": cpu_model()}
        if args.dtype == "f32" and not args.no_topk:
            # the oracle's top-k sorts; time it on the first 2^24 elements only and say so
            ns = min(D, 1 << 24)
            ks = -(-ns // 1000)
            Gs, Rs = Gn[:ns].copy(), to_np(ring[(t + 1) % 3])[:ns].copy()
            c3 = time.perf_counter()
            oracle.topk(Gs, Rs, ks)
            c4 = time.perf_counter()
            out["cpu_baseline"]["topk_sample"] = {
                "elements": ns, "k": ks, "us": round((c4 - c3) * 1e6),
                "note": "top-k oracle (full sort) on the first %d elements of the same gradient" % ns}

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
