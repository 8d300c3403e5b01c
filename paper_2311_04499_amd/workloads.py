"""Seeded synthetic gradient sets shaped like the DNNs the method is evaluated on.

This module holds NO arithmetic of the compression method: only tensor-shape
lists and random value generators.  It is the one module that both the CPU
oracle's tests and the HIP path's tests/benchmark draw inputs from, so both
sides see identical bits.  Values stand in for real training gradients (the
datasets and trained models of the paper's evaluation are not used): the path
is value-agnostic except for the top-k contrast, which only sees the
distribution.

Every generator takes an explicit integer seed derived from
(config id, worker, step) and a torch device; a CPU generator and a GPU
generator give different streams, so a test generates once and hands the same
tensor (copied) to both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import torch

Shape = Tuple[int, ...]


def _numel(shape: Shape) -> int:
    n = 1
    for d in shape:
        n *= d
    return n


# ---------------------------------------------------------------- shape lists

def tiny_mlp_shapes() -> List[Shape]:
    return [(1024, 512), (512,), (512, 256), (256,), (256, 10), (10,)]


def resnet50_shapes() -> List[Shape]:
    shapes: List[Shape] = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            shapes += [(planes, inplanes, 1, 1), (planes,), (planes,),
                       (planes, planes, 3, 3), (planes,), (planes,),
                       (planes * 4, planes, 1, 1), (planes * 4,), (planes * 4,)]
            if b == 0:
                shapes += [(planes * 4, inplanes, 1, 1), (planes * 4,), (planes * 4,)]
            inplanes = planes * 4
    shapes += [(1000, 2048), (1000,)]
    return shapes


def vgg19_shapes() -> List[Shape]:
    cfg = [64, 64, 128, 128, 256, 256, 256, 256, 512, 512, 512, 512, 512, 512, 512, 512]
    shapes: List[Shape] = []
    cin = 3
    for cout in cfg:
        shapes += [(cout, cin, 3, 3), (cout,)]
        cin = cout
    shapes += [(4096, 25088), (4096,), (4096, 4096), (4096,), (1000, 4096), (1000,)]
    return shapes


def bert_base_shapes() -> List[Shape]:
    h, ffn = 768, 3072
    shapes: List[Shape] = [(30522, h), (512, h), (2, h), (h,), (h,)]
    for _ in range(12):
        for _ in range(4):                      # query, key, value, attention output
            shapes += [(h, h), (h,)]
        shapes += [(h,), (h,)]                  # attention LayerNorm
        shapes += [(ffn, h), (ffn,), (h, ffn), (h,)]
        shapes += [(h,), (h,)]                  # output LayerNorm
    shapes += [(h, h), (h,)]                    # pooler
    return shapes


def gpt2_medium_shapes() -> List[Shape]:
    d, ffn = 1024, 4096
    shapes: List[Shape] = [(50257, d), (1024, d)]
    for _ in range(24):
        shapes += [(d,), (d,), (d, 3 * d), (3 * d,), (d, d), (d,),
                   (d,), (d,), (d, ffn), (ffn,), (ffn, d), (d,)]
    shapes += [(d,), (d,)]
    return shapes


# ---------------------------------------------------------------- workloads

@dataclass
class Workload:
    cfg_id: int
    name: str
    shapes: List[Shape]
    shard_elems: int
    n_workers: int
    K: int
    iterations: int
    dist: str                 # "normal" | "normal_fan_in" | "student_t3" | "bert"
    scale: float = 1e-3
    numel: List[int] = field(init=False)

    def __post_init__(self):
        self.numel = [_numel(s) for s in self.shapes]

    @property
    def D(self) -> int:
        return sum(self.numel)


def config(cfg_id: int) -> Workload:
    """The five benchmark configurations (1-based, in the order they are listed)."""
    if cfg_id == 1:
        return Workload(1, "tiny_mlp", tiny_mlp_shapes(), 4096, 4, 4, 8, "normal")
    if cfg_id == 2:
        return Workload(2, "resnet50", resnet50_shapes(), 65536, 8, 4, 50, "normal_fan_in")
    if cfg_id == 3:
        return Workload(3, "vgg19", vgg19_shapes(), 1 << 20, 16, 8, 50, "student_t3")
    if cfg_id == 4:
        # K = ceil(CCR) with CCR = 6
        return Workload(4, "bert_base", bert_base_shapes(), 1 << 18, 32, 6, 100, "bert")
    if cfg_id == 5:
        return Workload(5, "gpt2_medium", gpt2_medium_shapes(), 1 << 20, 64, 16, 100, "normal")
    raise ValueError("cfg_id must be 1..5")


def seed_for(cfg_id: int, worker: int, step: int, stream: int = 0) -> int:
    """A fixed, collision-free mixing of the four small integers into one seed."""
    return ((cfg_id * 1_000_003 + worker) * 1_000_033 + step) * 16 + stream


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _student_t3(n: int, device, g: torch.Generator, chunk: int = 1 << 26) -> torch.Tensor:
    """Student-t with 3 degrees of freedom: z / sqrt(chi2_3 / 3)."""
    out = torch.empty(n, dtype=torch.float32, device=device)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        z = torch.randn(m, generator=g, device=device)
        chi = torch.randn(3, m, generator=g, device=device).square_().sum(0)
        out[lo:lo + m] = z / torch.sqrt(chi / 3.0)
    return out


def gradient(wl: Workload, worker: int, step: int, device="cpu",
             dtype: torch.dtype = torch.float32) -> torch.Tensor:
    """One worker's flat gradient arena [D] for one iteration."""
    g = _gen(device, seed_for(wl.cfg_id, worker, step))
    D = wl.D
    if wl.dist == "student_t3":
        x = _student_t3(D, device, g).mul_(wl.scale)
    else:
        x = torch.randn(D, generator=g, device=device, dtype=torch.float32).mul_(wl.scale)
    if wl.dist == "normal_fan_in":
        off = 0
        for shape, n in zip(wl.shapes, wl.numel):
            fan_in = _numel(shape[1:]) if len(shape) > 1 else 1
            if fan_in > 1:
                x[off:off + n].mul_(1.0 / math.sqrt(fan_in))
            off += n
    elif wl.dist == "bert":
        # word-embedding gradient: 99% of the rows are exactly zero, the
        # touched rows are N(0, 1e-2); everything else stays N(0, 1e-3)
        rows, h = wl.shapes[0]
        emb = x[: rows * h].view(rows, h)
        keep = torch.rand(rows, generator=g, device=device) < 0.01
        emb.mul_(10.0)
        emb.mul_(keep.to(torch.float32).unsqueeze(1))
    return x.to(dtype) if dtype != torch.float32 else x


def payload_rows(wl: Workload, n_rows: int, n_elems: int, step: int, device="cpu",
                 dtype: torch.dtype = torch.float32, first_worker: int = 1) -> torch.Tensor:
    """Packed payloads [n_rows, n_elems] of the other workers, drawn directly at
    packed shape with the workload's dense-tensor distribution (used where
    running every worker's full compress would need N full arenas)."""
    out = torch.empty(n_rows, n_elems, dtype=dtype, device=device)
    for r in range(n_rows):
        g = _gen(device, seed_for(wl.cfg_id, first_worker + r, step, stream=1))
        if wl.dist == "student_t3":
            row = _student_t3(n_elems, device, g).mul_(wl.scale)
        else:
            row = torch.randn(n_elems, generator=g, device=device,
                              dtype=torch.float32).mul_(wl.scale)
        out[r] = row.to(dtype)
    return out


def integer_valued(n: int, seed: int, lo: int = -1000, hi: int = 1000, device="cpu") -> torch.Tensor:
    """fp32 tensor of small integers: sums of these are exact in fp32, which
    lets tests state conservation laws with == instead of a tolerance."""
    g = _gen(device, seed)
    return torch.randint(lo, hi + 1, (n,), generator=g, device=device).to(torch.float32)


def scaled_down(wl: Workload, numel: Sequence[int], shard_elems: int) -> Workload:
    """Same recipe on a smaller tensor list (for tests that must finish in seconds)."""
    w = Workload(wl.cfg_id, wl.name + "_small", [(int(n),) for n in numel], shard_elems,
                 wl.n_workers, wl.K, wl.iterations, "normal" if wl.dist in ("bert", "normal_fan_in") else wl.dist,
                 wl.scale)
    return w
