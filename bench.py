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
HIP-event duration, against the 8 TB/s peak), `kernels` (both), `configs` (the other
benchmark configurations, briefly), `median_sharding` (the same workload under the
paper's own sharding rule), `host_us_per_call`, the contrast kernels, the streamed
(per-bucket / overlapped) measurements and `cpu_baseline` (the CPU oracle on one full
iteration, one thread and all cores).  The line is a digest (about 2.5 KB); every
measurement in full goes to the file named by --details.  `--gpus N` with N > 1 is
refused: this build is a single-GPU path with no collectives.
"""
import argparse
import json
import os
import re
import statistics
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
    ap.add_argument("--shard-elems", type=int, default=0,
                    help="fixed-size shards of this many elements instead of the configuration's own")
    ap.add_argument("--row-align", type=int, default=1024,
                    help="receive rows start on multiples of this many elements (default 1024)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-topk", action="store_true")
    ap.add_argument("--no-probes", action="store_true")
    ap.add_argument("--no-streamed", action="store_true",
                    help="skip the per-bucket / HIP-graph / overlap measurements")
    ap.add_argument("--side-streams", type=int, default=3,
                    help="streams the per-bucket launches are dealt out to in the streamed section (default 3)")
    ap.add_argument("--details", default=os.path.join(ROOT, "gpurun_out", "bench_details.json"),
                    help="file that receives every measurement in full (the stdout line is a digest)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other configurations, the median-sharding run and the host-cost figures")
    return ap.parse_args()


def read_profile(kernel: str, workload: str):
    """(HBM bytes per launch, the kernel's average duration in us when they were taken, file) from the
    committed rocprofv3 --pmc summary, if any."""
    rel = os.path.join("profiles", f"{kernel}_{workload}_pmc.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None, None
    text = open(path).read()
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
    d = re.search(r"^profiled_avg_launch_us:\s*([0-9.eE+]+)", text, re.M)
    return (float(m.group(1)) if m else None), (float(d.group(1)) if d else None), rel


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


DTYPES = {  # name -> (gradient/dense, residual, payload) torch dtype names and the plan's code name
    "f32": ("float32", "float32", "float32", "COVAP_F32"),
    "bf16": ("bfloat16", "bfloat16", "bfloat16", "COVAP_BF16"),
    "bf16_res32": ("bfloat16", "float32", "bfloat16", "COVAP_BF16_RES32"),
    "f32_pay16": ("float32", "float32", "float16", "COVAP_F32_PAY16"),
}


class Run:
    """One workload resident in HBM: plan, gradient ring, residual, receive rows, dense result."""

    def __init__(self, torch, B, workloads, cfg, dtype, shard_mode, dev="cuda:0", ring=3, row_align=1024,
                 shard_elems=0):
        self.torch, self.B = torch, B
        self.wl = wl = workloads.config(cfg)
        if shard_elems:
            wl.shard_elems = shard_elems
        t, r, p, code = DTYPES[dtype]
        self.tdtype, self.rdtype, self.pdtype = getattr(torch, t), getattr(torch, r), getattr(torch, p)
        self.esz, self.rsz, self.psz = (torch.empty(0, dtype=d).element_size() for d in (self.tdtype, self.rdtype, self.pdtype))
        self.dtype, self.shard_mode = dtype, shard_mode
        self.plan = B.covap_plan(wl.numel, wl.shard_elems, wl.K, dtype=getattr(B, code),
                                 mode=B.COVAP_SHARD_FIXED if shard_mode == "fixed" else B.COVAP_SHARD_MEDIAN)
        self.D, self.N, self.K = self.plan.total_elems, wl.n_workers, wl.K
        self.stride = (self.plan.packed_elems_max + row_align - 1) // row_align * row_align   # default: 2 KiB boundaries at least
        self.ring = [workloads.gradient(wl, 0, i, dev, self.tdtype) for i in range(ring)]
        if self.D > wl.D:    # median sharding pads every communication tensor to a 1 KiB boundary of the arena
            self.ring = [torch.cat([g, g.new_zeros(self.D - wl.D)]) for g in self.ring]
        self.residual = torch.zeros(self.D, dtype=self.rdtype, device=dev)
        self.recv = torch.empty(self.N, self.stride, dtype=self.pdtype, device=dev)
        if self.N > 1:
            self.recv[1:] = workloads.payload_rows(wl, self.N - 1, self.stride, 0, dev, self.pdtype)
        self.dense = torch.empty(self.D, dtype=self.tdtype, device=dev)
        torch.cuda.synchronize()

    def compress(self, t, stream=None, bucket=-1, max_workgroups=None):
        self.B.covap_compress(self.plan, t, self.ring[t % len(self.ring)], self.residual, self.recv[0],
                              stream=stream, bucket=bucket, max_workgroups=max_workgroups)

    def decompress(self, t, stream=None, bucket=-1):
        self.B.covap_decompress(self.plan, t, self.recv, self.dense, n_workers=self.N, stride_elems=self.stride,
                                stream=stream, bucket=bucket)

    def timed_steps(self, steps, warmup):
        """Exactly `steps` steps after `warmup` untimed ones, HIP events around every kernel (recorded on
        the stream the kernels are launched on).  Returns per-kernel times (ms) and the wall clock."""
        torch = self.torch
        stream = torch.cuda.current_stream()
        for t in range(warmup):
            self.compress(t, stream)
            self.decompress(t, stream)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        for i in range(steps):
            t = warmup + i
            ev[i][0].record(stream)
            self.compress(t, stream)
            ev[i][1].record(stream)
            self.decompress(t, stream)
            ev[i][2].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - wall0
        tc = [e[0].elapsed_time(e[1]) for e in ev]
        td = [e[1].elapsed_time(e[2]) for e in ev]
        ts = list(range(warmup, warmup + steps))
        P_avg = sum(self.plan.packed_elems(t) for t in ts) / len(ts)
        bytes_c = self.esz * self.D + self.psz * P_avg + self.rsz * 2 * self.D   # read G, read R, write R, write packed
        bytes_d = self.psz * self.N * P_avg + self.esz * self.D                   # read N rows, write dense
        return tc, td, wall, bytes_c, bytes_d

    def host_us_per_call(self, reps=64):
        """Host time of one covap_compress / covap_decompress call (arguments, launch geometry, enqueue),
        measured over `reps` back-to-back calls each; the GPU runs behind."""
        torch = self.torch
        stream = torch.cuda.current_stream()
        out = {}
        for name, fn in (("compress", self.compress), ("decompress", self.decompress)):
            fn(0, stream)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for t in range(reps):
                fn(t, stream)
            out[name] = round((time.perf_counter() - t0) * 1e6 / reps, 2)
            torch.cuda.synchronize()
        return out


def kernel_stats(ts_ms, nbytes):
    ys = sorted(ts_ms)
    avg = sum(ys) / len(ys)
    pct = lambda q: round(ys[min(len(ys) - 1, int(q * len(ys)))] * 1e3, 2)
    gbs = nbytes / (avg * 1e-3) / 1e9
    return {"avg_us": round(avg * 1e3, 2), "p10_us": pct(0.1), "median_us": pct(0.5), "p90_us": pct(0.9),
            "algorithmic_bytes": round(nbytes), "GB/s": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4)}


def brief(run, steps, warmup):
    """ms/step and per-kernel fractions of one configuration, for the `configs` block."""
    tc, td, wall, bc, bd = run.timed_steps(steps, warmup)
    kc, kd = kernel_stats(tc, bc), kernel_stats(td, bd)
    return {"workload": f"cfg{run.wl.cfg_id}:{run.wl.name}", "dtype": run.dtype, "sharding": run.shard_mode,
            "elements": run.D, "shards": run.plan.num_shards, "n_workers": run.N, "K": run.K, "steps": steps,
            "ms_per_step": round(wall * 1e3 / steps, 4),
            "grad_GB/s": round(run.esz * run.D / (wall / steps) / 1e9, 1),
            "compress": {k: kc[k] for k in ("avg_us", "p10_us", "median_us", "p90_us", "GB/s", "frac")},
            "decompress": {k: kd[k] for k in ("avg_us", "p10_us", "median_us", "p90_us", "GB/s", "frac")}}


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
    run = Run(torch, B, workloads, args.config, args.dtype, args.shard_mode, dev, row_align=args.row_align,
              shard_elems=args.shard_elems)
    wl, plan, D, N, K = run.wl, run.plan, run.D, run.N, run.K
    esz, stride, ring, residual, recv, dense = run.esz, run.stride, run.ring, run.residual, run.recv, run.dense
    stream = torch.cuda.current_stream()

    # ---- timed region: exactly `steps` steps, HIP events around every kernel
    tc, td, wall, bytes_c, bytes_d = run.timed_steps(args.steps, args.warmup)
    ms_step = wall * 1e3 / args.steps
    tc_avg, td_avg = sum(tc) / len(tc), sum(td) / len(td)
    grad_gbs = esz * D / (ms_step * 1e-3) / 1e9
    hbm_gbs = (bytes_c + bytes_d) / (ms_step * 1e-3) / 1e9

    dominant = ("covap_decompress", td_avg, bytes_d) if td_avg >= tc_avg else \
               ("covap_compress", tc_avg, bytes_c)
    ach = dominant[2] / (dominant[1] * 1e-3) / 1e9
    # Counter traffic is not measured by this run: it comes from the committed rocprofv3 --pmc summary of
    # the same command (default element type, sharding and knobs only), and is dropped when this run's
    # kernel time is more than 5 % away from the time the kernel took when the counters were read.
    traffic, traffic_source = None, None
    if args.dtype == "f32" and args.shard_mode == "fixed" and not args.tune:
        tb, prof_us, rel = read_profile(dominant[0], wl.name)
        if tb is not None and prof_us is not None and abs(dominant[1] * 1e3 - prof_us) <= 0.05 * prof_us:
            traffic, traffic_source = tb, rel
    roofline = {"bound": "hbm", "kernel": dominant[0], "achieved": round(ach, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                "bytes_per_launch": round(dominant[2]), "avg_launch_us": round(dominant[1] * 1e3, 2)}

    kernels = {"covap_compress": kernel_stats(tc, bytes_c), "covap_decompress": kernel_stats(td, bytes_d)}

    out = {
        "metric": "compress+decompress GB/s of gradient processed", "value": round(grad_gbs, 2),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"cfg{wl.cfg_id}:{wl.name}", "elements": D, "shard_elems": wl.shard_elems,
                   "n_workers": N, "K": K, "mode": "payload", "sharding": args.shard_mode,
                   "shards": plan.num_shards},
        "hbm_GB/s": round(hbm_gbs, 1), "hbm_frac": round(hbm_gbs / HBM_PEAK_GBS, 4),
        "target_hbm_frac_0.70_met": bool(hbm_gbs / HBM_PEAK_GBS >= 0.70),
        "overhead_us_per_iter": round(ms_step * 1e3, 1),
        "roofline": roofline, "kernels": kernels,
    }

    def timed_us(fn, reps=10, warm=2):
        for t in range(warm):
            fn(t)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for t in range(reps):
            fn(t)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    # ---- achievable streaming rate in the same run (context for the fraction)
    if not args.no_probes:
        nb_ = min(D * esz, 1 << 31) // 16 * 16
        a = dense.view(torch.uint8)[:nb_]
        b = ring[0].view(torch.uint8)[:nb_]
        us = timed_us(lambda t: B.covap_probe_copy(a, b, nb_, stream=stream), reps=20, warm=3)
        out["probe_copy_GB/s"] = round(2 * nb_ / (us * 1e-6) / 1e9, 1)
        if args.dtype == "f32":
            # a = b + s*c: the two-reads-one-write shape of compress without its index work
            nt = nb_ // 4
            ta, tb_, tc_ = dense[:nt], ring[0][:nt], ring[1][:nt]
            us = timed_us(lambda t: B.covap_probe_triad(ta, tb_, tc_, 0.5, nt, stream=stream), reps=20, warm=3)
            out["probe_triad_GB/s"] = round(3 * nb_ / (us * 1e-6) / 1e9, 1)

    # ---- top-k contrast on the same gradient buffers
    if not args.no_topk and args.dtype == "f32":
        try:
            k = -(-D // 1000)                            # ceil(0.1% of D)
            ws = torch.empty(B.topk_workspace_bytes(D), dtype=torch.uint8, device=dev)
            vals = torch.empty(k, dtype=torch.float32, device=dev)
            idx = torch.empty(k, dtype=torch.int32, device=dev)
            res2 = torch.zeros(D, dtype=torch.float32, device=dev)
            topk_us = timed_us(lambda t: B.topk_compress(ring[t % 3], res2, k, vals, idx, ws, stream=stream),
                               reps=max(5, min(args.steps, 20)), warm=3)
            ratio = topk_us / (tc_avg * 1e3)
            out["topk"] = {"k": k, "us_per_iter": round(topk_us, 1),
                           "vs_covap_compress": round(ratio, 2),
                           "vs_covap_compress_plus_decompress": round(topk_us / (ms_step * 1e3), 2),
                           # the other half of the stated goal: compression overhead at least 10x below top-k's
                           "target_10x_below_topk_met": bool(ratio >= 10.0)}
            # the ratio of the paper's Table II (k = 1 %), for context beside the 0.1 % this benchmark is quoted on
            k1 = -(-D // 100)
            vals1 = torch.empty(k1, dtype=torch.float32, device=dev)
            idx1 = torch.empty(k1, dtype=torch.int32, device=dev)
            res2.zero_()                                 # its own error-feedback history, from the start
            us1 = timed_us(lambda t: B.topk_compress(ring[t % 3], res2, k1, vals1, idx1, ws, stream=stream),
                           reps=max(5, min(args.steps, 20)), warm=3)
            out["topk"]["at_1_percent"] = {"k": k1, "us_per_iter": round(us1, 1),
                                           "vs_covap_compress": round(us1 / (tc_avg * 1e3), 2)}
            del ws, vals, idx, res2, vals1, idx1
        except B.CovapError as e:
            out["topk"] = {"error": str(e)}

    # ---- Random-k (k = 1 %) and FP16 contrast kernels on the same gradient buffers
    if not args.no_topk and args.dtype == "f32":
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
                us = timed_us(lambda t: B.sparse_decompress_sorted(sv, si, dense, stream=stream), reps=20, warm=5)
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
        us = timed_us(lambda t: B.covap_compress_aliased(plan, t, acc_buf, recv[0], stream=stream), reps=2 * K, warm=K)
        P_period = sum(plan.packed_elems(t) for t in range(K)) / K
        out["aliased_compress"] = {"us_per_iter": round(us, 2), "algorithmic_bytes": round(3 * esz * P_period),
                                   "GB/s": round(3 * esz * P_period / (us * 1e-6) / 1e9, 1)}
        if "topk" in out and "us_per_iter" in out["topk"]:
            out["aliased_compress"]["topk_over_aliased"] = round(out["topk"]["us_per_iter"] / us, 1)
        del acc_buf

    # ---- the step after a sum-AllReduce (Sec. II-A, III-B): the collective has added the rows; one summed row
    # comes in, summed / N goes out.  What one GPU of a real job runs per iteration is compress + this, not the
    # N-row mean that `value` prices.
    P_period = sum(plan.packed_elems(t) for t in range(K)) / K
    pay_esz = recv.element_size()
    us = timed_us(lambda t: B.covap_decompress_reduced(plan, t, recv[min(1, N - 1)], dense, N, stream=stream), reps=2 * K, warm=K)
    red_bytes = pay_esz * P_period + esz * D
    out["allreduce_form"] = {"decompress_reduced_us": round(us, 2), "algorithmic_bytes": round(red_bytes),
                             "GB/s": round(red_bytes / (us * 1e-6) / 1e9, 1),
                             "frac": round(red_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                             "compress_plus_decompress_reduced_us": round(tc_avg * 1e3 + us, 1),
                             "gradient_GB/s": round(esz * D / ((tc_avg * 1e3 + us) * 1e-6) / 1e9, 1)}

    # ---- per-bucket streamed mode: one launch per communication bucket, as a DDP hook
    # would issue them while backward is still running (Sec. II-B); eager launches,
    # HIP graphs (one per residue of the step), and overlap with a synthetic backward
    if not args.no_streamed:
        out["streamed"] = streamed(torch, B, run, ms_step, args)

    # ---- the other benchmark configurations, the paper's sharding rule on this one, host cost per call
    if not args.no_configs:
        del ring, residual, recv, dense
        host = {args.shard_mode: run.host_us_per_call()}
        steps_b, warm_b = max(5, min(args.steps, 20)), 3
        if args.shard_mode == "fixed" and args.dtype == "f32":
            mrun = Run(torch, B, workloads, args.config, args.dtype, "median", dev)
            ms = brief(mrun, steps_b, warm_b)
            host["median"] = mrun.host_us_per_call()
            _, _, _, _, launches, groups = mrun.plan.trace(0, -1, 256, False)
            ms["launches_per_call"] = launches
            ms["communication_tensors"] = mrun.plan.num_buckets
            out["median_sharding"] = ms
            del mrun
        out["host_us_per_call"] = host
        cfgs = []
        for cfg, dt in ((1, "f32"), (2, "f32"), (3, "f32"), (4, "f32"), (4, "bf16")):
            if cfg == args.config and dt == args.dtype:
                continue
            r = Run(torch, B, workloads, cfg, dt, "fixed", dev)
            cfgs.append(brief(r, steps_b, warm_b))
            del r
        out["configs"] = cfgs

    # ---- CPU oracle on a bounded sample of the same workload (reported, not a target)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(torch, run, args)

    # The one line on stdout stays short (a record keeper may keep only the end of a run's output); everything
    # measured goes, in full, to a file beside it.
    details = args.details
    try:
        os.makedirs(os.path.dirname(details) or ".", exist_ok=True)
        with open(details, "w") as f:
            json.dump(out, f, indent=1)
    except OSError:
        details = None
    print(json.dumps(compact(out, details), separators=(",", ":")), flush=True)


def compact(out, details):
    """The contract's fields in full, the rest boiled down to the figures that matter."""
    line = {k: out[k] for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                                "higher_is_better", "scaling", "vs_baseline", "dtype", "data")}
    c = out["config"]
    line["config"] = {k: c[k] for k in ("workload", "elements", "shard_elems", "n_workers", "K", "mode", "sharding")}
    r = out["roofline"]
    line["roofline"] = {k: r[k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "traffic",
                                          "traffic_source", "avg_launch_us")}
    line["hbm_frac"] = out["hbm_frac"]
    line["target_hbm_frac_0.70_met"] = out["target_hbm_frac_0.70_met"]
    line["kernels"] = {k[6:]: {"avg_us": v["avg_us"], "frac": v["frac"]} for k, v in out["kernels"].items()}
    if "cpu_baseline" in out:
        b = out["cpu_baseline"]
        line["cpu_baseline"] = {k: b[k] for k in ("value", "unit", "cores", "kind", "sample")}
        if "all_cores" in b:
            a = b["all_cores"]
            line["cpu_baseline"]["all_cores"] = {"value": a["value"], "cores": a["cores"],
                                                 "bit_identical": a["bit_identical_to_single_thread"]}
    if "topk" in out and "us_per_iter" in out["topk"]:
        t = out["topk"]
        line["topk"] = {k: t[k] for k in ("us_per_iter", "vs_covap_compress", "target_10x_below_topk_met",
                                          "decompress_us_per_iter") if k in t}
        if "at_1_percent" in t:
            line["topk"]["us_per_iter_at_1_percent"] = t["at_1_percent"]["us_per_iter"]
    if "aliased_compress" in out:
        a = out["aliased_compress"]
        line["aliased_compress"] = {k: a[k] for k in ("us_per_iter", "topk_over_aliased") if k in a}
    if "allreduce_form" in out:
        a = out["allreduce_form"]
        line["allreduce_form"] = {k: a[k] for k in ("decompress_reduced_us", "frac", "compress_plus_decompress_reduced_us")}
    if "streamed" in out:
        st = out["streamed"]
        line["streamed"] = {"buckets": st["buckets"], "eager_us_per_step": st["eager_us_per_step"],
                            "side_streams_us_per_step": st.get("eager_side_streams_us_per_step"),
                            "graph_us_per_step": st.get("graph_us_per_step"),
                            "graph_side_streams_us_per_step": st.get("graph_side_streams_us_per_step")}
        brief_ov = lambda v: {k: v[k] for k in ("hidden_frac", "exposed_us", "sync_only_us", "compress_us", "backward_us")}
        if "overlap" in st:
            line["streamed"]["overlap"] = dict(brief_ov(st["overlap"]), variant=st["overlap"]["variant"])
            for name in ("mfma_only_handover_every_8", "gemm_aliased_handover_every_8"):
                if name in st["overlap_variants"]:
                    line["streamed"][name] = brief_ov(st["overlap_variants"][name])
        elif "overlap_error" in st:
            line["streamed"]["overlap_error"] = st["overlap_error"][:80]
    if "configs" in out:
        line["configs"] = [{"workload": c["workload"], "dtype": c["dtype"], "ms_per_step": c["ms_per_step"],
                            "compress_frac": c["compress"]["frac"], "decompress_frac": c["decompress"]["frac"]}
                           for c in out["configs"]]
    if "median_sharding" in out:
        m = out["median_sharding"]
        line["median_sharding"] = {"ms_per_step": m["ms_per_step"], "compress_frac": m["compress"]["frac"],
                                   "decompress_frac": m["decompress"]["frac"], "launches_per_call": m["launches_per_call"]}
    if "host_us_per_call" in out:
        line["host_us_per_call"] = out["host_us_per_call"]
    line["details"] = os.path.relpath(details, ROOT) if details else None
    return line


def streamed(torch, B, run, ms_step, args):
    plan, N, K, stride = run.plan, run.N, run.K, run.stride
    ring, residual, recv, dense = run.ring, run.residual, run.recv, run.dense
    dev = recv.device
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
    _, eager_wall_us = timed(per_bucket, reps)
    sres = {"buckets": nb, "launches_per_step": 2 * nb,
            "eager_us_per_step": round(eager_wall_us, 1),
            "whole_arena_us_per_step": round(ms_step * 1e3, 1)}

    # the same launches dealt out to a few streams (bucket b on stream b mod 3 by default; a bucket's decompress
    # follows its compress on the same stream): the next bucket's kernel starts while the last one's final waves
    # drain (measured: 1 stream 2.06 ms with the fork and join, 2: 1.88, 3: 1.81, 4: 1.85, 8: 1.84 ms)
    try:
        n_side = max(1, args.side_streams)
        pair = [torch.cuda.Stream() for _ in range(n_side)]
        fork, joins = torch.cuda.Event(), [torch.cuda.Event() for _ in range(n_side)]

        def per_bucket_two_streams(t):
            main = torch.cuda.current_stream()
            fork.record(main)
            for st in pair:
                st.wait_event(fork)
            for b in range(nb):
                B.covap_compress(plan, t, ring[0], residual, recv[0], bucket=b, stream=pair[b % n_side])
            for b in range(nb):
                B.covap_decompress(plan, t, recv, dense, n_workers=N, stride_elems=stride, bucket=b,
                                   stream=pair[b % n_side])
            for st, ev in zip(pair, joins):
                ev.record(st)
                main.wait_event(ev)

        per_bucket_two_streams(0)
        _, two_wall_us = timed(per_bucket_two_streams, reps)
        sres["eager_side_streams"] = n_side
        sres["eager_side_streams_us_per_step"] = round(two_wall_us, 1)
    except Exception as e:                              # reported, never hidden
        sres["side_streams_error"] = repr(e)[:200]

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
    # the same graphs with the launches dealt out to the side streams inside the capture (fork and join events
    # become graph edges, so buckets on different streams may run side by side on replay)
    if "eager_side_streams_us_per_step" in sres:
        try:
            graphs2 = []
            side2 = torch.cuda.Stream()
            for r in range(K):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side2):
                    per_bucket_two_streams(r)
                graphs2.append(g)
            for g in graphs2:
                g.replay()
            _, graph2_wall_us = timed(lambda t: graphs2[t % K].replay(), reps)
            sres["graph_side_streams_us_per_step"] = round(graph2_wall_us, 1)
            del graphs2
        except Exception as e:                          # reported, never hidden
            sres["graph_side_streams_error"] = repr(e)[:200]

    # Overlap (Sec. II-B: compression is meant to hide behind backward propagation).  The stand-in for
    # backward is one bf16 GEMM (4096^3, the library's own kernel) per bucket on the main stream; compress of
    # bucket b is issued on a side stream once "its gradient is ready" (an event after GEMM b).  Every figure
    # is the median over paired repetitions, each taken right after a plain backward pass, so that clock and
    # temperature drift (a few per cent of the 6 ms pass, as much as what is measured) cancel:
    #   exposed        = overlapped pass - backward pass
    #   sync_only      = the same pass with the events and the cross-stream waits but no compress
    #   hidden_frac    = 1 - exposed / compress alone
    try:
        m = 4096
        xa = torch.randn(m, m, device=dev, dtype=torch.bfloat16)
        xb = torch.randn(m, m, device=dev, dtype=torch.bfloat16)
        xc = torch.empty(m, m, device=dev, dtype=torch.bfloat16)
        spin_out = torch.empty(256 * 256, device=dev)
        side = torch.cuda.Stream()
        ready = [torch.cuda.Event() for _ in range(nb)]
        done = torch.cuda.Event()
        gemm = lambda: torch.mm(xa, xb, out=xc)
        # matrix-core work on registers only, the occupancy of the GEMM above (one 256-thread workgroup and
        # 64 KiB of LDS per compute unit), about as long: what is exposed next to it is not memory contention
        spin = lambda: B.covap_probe_mfma(spin_out, 256, 3000, 65536)

        aliased_ok = run.dtype in ("f32", "bf16")
        acc_buf = ring[1].clone() if aliased_ok else None

        def passes(work, group, cap, compress=True, aliased=False):
            def one(t, b, st):
                if aliased:   # the producer accumulates into acc_buf; only the sent shards are moved and cleared
                    B.covap_compress_aliased(plan, t, acc_buf, recv[0], bucket=b, stream=st)
                else:
                    B.covap_compress(plan, t, ring[0], residual, recv[0], bucket=b, stream=st, max_workgroups=cap)

            def backward_only(t):
                for b in range(nb):
                    work()

            def compress_only(t):
                for b in range(nb):
                    one(t, b, None)

            def overlapped(t):
                for b in range(nb):
                    work()
                    if b % group == group - 1 or b == nb - 1:      # one hand-over per `group` buckets
                        ready[b].record()
                        side.wait_event(ready[b])
                        if compress:
                            for bb in range(b - b % group, b + 1):
                                one(t, bb, side)
                done.record(side)
                torch.cuda.current_stream().wait_event(done)
            return backward_only, compress_only, overlapped

        def paired(work, group=1, cap=None, pairs=9, aliased=False):
            bo, co, ov = passes(work, group, cap, aliased=aliased)
            _, _, sync = passes(work, group, cap, compress=False)
            for f in (bo, co, ov, sync):
                f(0)
            d_ov, d_sync, t_bw, t_co = [], [], [], []
            for i in range(pairs):
                bw, _ = timed(bo, 1)
                o, _ = timed(ov, 1)
                bw2, _ = timed(bo, 1)
                s, _ = timed(sync, 1)
                c, _ = timed(co, 1)
                d_ov.append(o - bw)
                d_sync.append(s - bw2)
                t_bw.append(bw)
                t_co.append(c)
            med = statistics.median
            exposed, co_us = med(d_ov), med(t_co)
            return {"backward_us": round(med(t_bw), 1), "compress_us": round(co_us, 1),
                    "exposed_us": round(exposed, 1), "sync_only_us": round(med(d_sync), 1),
                    "hidden_frac": round(1.0 - max(exposed, 0.0) / co_us, 3), "pairs": pairs,
                    "handover_every_buckets": group, "max_workgroups": cap, "aliased_residual": aliased}

        ov = {"gemm_per_bucket": paired(gemm), "gemm_handover_every_8": paired(gemm, group=8),
              "gemm_bounded_4096_workgroups": paired(gemm, cap=4096),
              "mfma_only_per_bucket": paired(spin), "mfma_only_handover_every_8": paired(spin, group=8)}
        if aliased_ok:
            ov["gemm_aliased_per_bucket"] = paired(gemm, aliased=True)
            ov["gemm_aliased_handover_every_8"] = paired(gemm, group=8, aliased=True)
        best = max(("gemm_per_bucket", "gemm_handover_every_8", "gemm_bounded_4096_workgroups"),
                   key=lambda k: ov[k]["hidden_frac"])
        sres["overlap"] = dict(ov[best], variant=best)
        sres["overlap_variants"] = ov
        del xa, xb, xc
    except Exception as e:
        sres["overlap_error"] = repr(e)[:200]
    return sres


def cpu_baseline(torch, run, args):
    """The oracle as it stands on one full iteration of the same workload: one thread (the primary
    figure), then the same C routines called on runs of whole shards from a thread pool over all cores
    (same per-element order, identical bits)."""
    import numpy as np
    import oracle
    wl, D, K, esz, psz = run.wl, run.D, run.K, run.esz, run.psz
    tab = oracle.plan_fixed(wl.numel, wl.shard_elems, (25 << 20) // esz) if args.shard_mode == "fixed" \
        else oracle.plan_median(wl.numel, (25 << 20) // esz, K, 0, 1024 // psz)
    t = args.warmup + args.steps
    to_np = lambda x: x.cpu().numpy() if x.dtype == torch.float32 else \
        x.cpu().view(torch.int16).numpy().view(np.uint16)
    # inputs are generated, never taken from the GPU path's outputs: a gradient, a residual
    # of the same scale, and the synthetic payload rows (row 0 is filled by the oracle itself)
    Gn = to_np(run.ring[t % 3])
    R0 = to_np(run.ring[(t + 1) % 3].to(run.rdtype)).copy()
    recv_n = to_np(run.recv).copy()
    recv_n[0] = 0
    out_n = np.empty(D, Gn.dtype)
    Rn = R0.copy()
    c0 = time.perf_counter()
    oracle.compress(tab, K, t, Gn, Rn, recv_n[0])
    c1 = time.perf_counter()
    oracle.decompress(tab, K, t, recv_n, out_n)
    c2 = time.perf_counter()
    res = {"value": round(esz * D / (c2 - c0) / 1e9, 4), "unit": "GB/s",
           "cores": 1, "kind": "oracle",
           "sample": "1 full iteration of the same workload (compress %.2f s + "
                     "decompress %.2f s), single thread" % (c1 - c0, c2 - c1),
           "compress_us_per_iter": round((c1 - c0) * 1e6),
           "decompress_us_per_iter": round((c2 - c1) * 1e6),
           "host_cpus": os.cpu_count(), "cpu_model": cpu_model()}
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
    if cores > 1:
        first = (recv_n[0].copy(), Rn.copy(), out_n.copy())
        Rn = R0.copy()
        recv_n[0] = 0
        a0 = time.perf_counter()
        oracle.compress(tab, K, t, Gn, Rn, recv_n[0], threads=cores)
        a1 = time.perf_counter()
        oracle.decompress(tab, K, t, recv_n, out_n, threads=cores)
        a2 = time.perf_counter()
        same = all(np.array_equal(x.view(np.uint8), y.view(np.uint8))
                   for x, y in zip(first, (recv_n[0], Rn, out_n)))
        res["all_cores"] = {"value": round(esz * D / (a2 - a0) / 1e9, 4), "unit": "GB/s", "cores": cores,
                            "kind": "oracle, the same C routines on runs of whole shards from a thread pool",
                            "compress_us_per_iter": round((a1 - a0) * 1e6),
                            "decompress_us_per_iter": round((a2 - a1) * 1e6),
                            "bit_identical_to_single_thread": bool(same)}
    if args.dtype == "f32" and not args.no_topk:
        # the oracle's top-k sorts; time it on the first 2^24 elements only and say so
        ns = min(D, 1 << 24)
        ks = -(-ns // 1000)
        Gs, Rs = Gn[:ns].copy(), to_np(run.ring[(t + 1) % 3])[:ns].copy()
        c3 = time.perf_counter()
        oracle.topk(Gs, Rs, ks)
        c4 = time.perf_counter()
        res["topk_sample"] = {
            "elements": ns, "k": ks, "us": round((c4 - c3) * 1e6),
            "note": "top-k oracle (full sort) on the first %d elements of the same gradient" % ns}
    return res


if __name__ == "__main__":
    main()
