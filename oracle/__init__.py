"""CPU oracle of the COVAP hot path -- TEST INFRASTRUCTURE, not product code.

Thin ctypes wrapper over ``covap_oracle.c`` (plain C, built with gcc).  Only
``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg
may import this package; the HIP library never does, and this package never
imports the HIP binding.  All arrays are numpy, host memory.

The arithmetic lives in the C file; this module only marshals arguments.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "covap_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None

_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)
_u16p = C.POINTER(C.c_uint16)
_u32p = C.POINTER(C.c_uint32)


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        L.orc_plan_offsets.restype = C.c_int64
        L.orc_plan_offsets.argtypes = [_i64p, C.c_int32, _i64p]
        L.orc_plan_fixed_shards.restype = C.c_int64
        L.orc_plan_fixed_shards.argtypes = [C.c_int64, C.c_int64, _i64p, _i64p]
        L.orc_plan_buckets.restype = C.c_int32
        L.orc_plan_buckets.argtypes = [_i64p, C.c_int64, C.c_int64, _i32p]
        L.orc_plan_median_parts.restype = C.c_int64
        L.orc_plan_median_parts.argtypes = [_i64p, C.c_int32, C.c_int64, C.c_int32, _i32p]
        L.orc_plan_median_layout.restype = C.c_int64
        L.orc_plan_median_layout.argtypes = [_i64p, C.c_int32, C.c_int64, C.c_int32, C.c_int64, C.c_int64,
                                             _i64p, _i64p, _i64p, _i32p, _i64p]
        L.orc_plan_even_slices.restype = C.c_int32
        L.orc_plan_even_slices.argtypes = [C.c_int64, C.c_int32, C.c_int64, _i64p]
        L.orc_selected.restype = C.c_int32
        L.orc_selected.argtypes = [C.c_int64, C.c_uint64, C.c_int32]
        L.orc_packed_end.restype = C.c_int64
        L.orc_packed_end.argtypes = [_i64p, C.c_int64, C.c_int32, C.c_uint64, C.c_int64]
        L.orc_plan_group_layers.restype = C.c_int32
        L.orc_plan_group_layers.argtypes = [_i64p, C.c_int32, C.c_int64, _i32p]
        L.orc_f32_to_bf16.restype = C.c_uint16
        L.orc_f32_to_bf16.argtypes = [C.c_float]
        L.orc_bf16_to_f32.restype = C.c_float
        L.orc_bf16_to_f32.argtypes = [C.c_uint16]
        for name, ptr in (("f32", _f32p), ("bf16", _u16p)):
            f = getattr(L, "orc_compress_" + name)
            f.restype = C.c_int64
            f.argtypes = [ptr, ptr, ptr, _i64p, _i64p, C.c_int64, C.c_int64, C.c_int32,
                          C.c_uint64, C.c_float, C.c_int64]
            g = getattr(L, "orc_decompress_" + name)
            g.restype = None
            g.argtypes = [ptr, C.c_int32, C.c_int64, ptr, _i64p, _i64p, C.c_int64, C.c_int64,
                          C.c_int32, C.c_uint64, C.c_int64]
        L.orc_compress_bf16_res32.restype = C.c_int64
        L.orc_compress_bf16_res32.argtypes = [_u16p, _f32p, _u16p, _i64p, _i64p, C.c_int64, C.c_int64,
                                              C.c_int32, C.c_uint64, C.c_float, C.c_int64]
        L.orc_compress_aliased.restype = C.c_int64
        L.orc_compress_aliased.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _i64p, _i64p, C.c_int64,
                                           C.c_int64, C.c_int32, C.c_uint64, C.c_int64]
        L.orc_topk_f32.restype = C.c_int32
        L.orc_topk_f32.argtypes = [_f32p, _f32p, C.c_int64, C.c_int64, C.c_float, _f32p, _u32p]
        L.orc_randk_f32.restype = C.c_int32
        L.orc_randk_f32.argtypes = [_f32p, _f32p, C.c_int64, _u32p, C.c_int64, C.c_float, _f32p]
        L.orc_f32_to_f16.restype = C.c_uint16
        L.orc_f32_to_f16.argtypes = [C.c_float]
        L.orc_f16_to_f32.restype = C.c_float
        L.orc_f16_to_f32.argtypes = [C.c_uint16]
        L.orc_compress_f32_pay16.restype = C.c_int64
        L.orc_compress_f32_pay16.argtypes = [_f32p, _f32p, _u16p, _i64p, _i64p, C.c_int64, C.c_int64,
                                             C.c_int32, C.c_uint64, C.c_float, C.c_int64]
        L.orc_decompress_pay16.restype = None
        L.orc_decompress_pay16.argtypes = [_u16p, C.c_int32, C.c_int64, _f32p, _i64p, _i64p, C.c_int64,
                                           C.c_int64, C.c_int32, C.c_uint64, C.c_int64]
        for name, pin, pout in (("f32", _f32p, _f32p), ("bf16", _u16p, _u16p), ("pay16", _u16p, _f32p)):
            f = getattr(L, "orc_unpack_mean_" + name)
            f.restype = None
            f.argtypes = [pin, C.c_int32, pout, _i64p, _i64p, C.c_int64, C.c_int64, C.c_int32, C.c_uint64, C.c_int64]
        L.orc_fp16_compress.restype = None
        L.orc_fp16_compress.argtypes = [_f32p, _f32p, C.c_int64, C.c_float, _u16p]
        L.orc_fp16_mean.restype = None
        L.orc_fp16_mean.argtypes = [_u16p, C.c_int32, C.c_int64, C.c_int64, _f32p]
        L.orc_sparse_mean.restype = None
        L.orc_sparse_mean.argtypes = [_f32p, _u32p, C.c_int32, C.c_int64, C.c_int64, C.c_int64, _f32p]
        L.orc_ratio_from_ccr.restype = C.c_int32
        L.orc_ratio_from_ccr.argtypes = [C.c_double, _i32p]
        L.orc_ef_coeff.restype = C.c_float
        L.orc_ef_coeff.argtypes = [C.c_float, C.c_uint64, C.c_uint64, C.c_float]
        _lib = L
    return _lib


def _p(a: np.ndarray, ptr):
    return a.ctypes.data_as(ptr)


def _ranges(tab: "ShardTable", lo: int, hi: int, threads: int):
    """[lo, hi) cut into runs of whole shards of about equal element counts, a few per thread."""
    if threads <= 1 or hi - lo <= 1:
        return [(lo, hi)]
    want = max(1, int(tab.len[lo:hi].sum()) // (4 * threads))
    cuts, acc = [lo], 0
    for s in range(lo, hi):
        acc += int(tab.len[s])
        if acc >= want and s + 1 < hi:
            cuts.append(s + 1)
            acc = 0
    cuts.append(hi)
    return list(zip(cuts[:-1], cuts[1:]))


def _run(calls, threads: int):
    """Run the C calls one after the other, or -- threads > 1 -- on a thread pool (ctypes
    releases the interpreter lock).  Every call covers its own run of whole shards and works
    out its own packed position, so the element-wise results do not depend on the split."""
    if threads <= 1 or len(calls) <= 1:
        return [f() for f in calls]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda f: f(), calls))


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    if a.dtype != dtype or not a.flags.c_contiguous:
        raise TypeError(f"expected C-contiguous {dtype}, got {a.dtype}")
    return a


# ------------------------------------------------------------------ planner

class ShardTable:
    """Shard list of one arena: off[s], len[s], bucket[s]; D elements in all.
    `align`: every sent shard starts at a multiple of this many elements in the
    packed layout (1 = plain concatenation)."""

    def __init__(self, off, length, bucket, D, tensor_offsets=None, align=1):
        self.off = np.ascontiguousarray(off, dtype=np.int64)
        self.len = np.ascontiguousarray(length, dtype=np.int64)
        self.bucket = np.ascontiguousarray(bucket, dtype=np.int32)
        self.D = int(D)
        self.tensor_offsets = tensor_offsets
        self.align = int(align)

    @property
    def n_shards(self) -> int:
        return int(self.off.shape[0])

    @property
    def n_buckets(self) -> int:
        return int(self.bucket[-1]) + 1 if self.n_shards else 0

    def bucket_range(self, b: int):
        """Shard range [lo, hi) of bucket b; b = -1 means every shard."""
        if b < 0:
            return 0, self.n_shards
        idx = np.nonzero(self.bucket == b)[0]
        return int(idx[0]), int(idx[-1]) + 1


def plan_fixed(tensor_numel, shard_elems: int, bucket_cap_elems: int) -> ShardTable:
    numel = np.ascontiguousarray(tensor_numel, dtype=np.int64)
    offs = np.zeros(max(len(numel), 1), dtype=np.int64)
    D = lib().orc_plan_offsets(_p(numel, _i64p), len(numel), _p(offs, _i64p))
    n = lib().orc_plan_fixed_shards(D, shard_elems, None, None)
    off = np.zeros(max(n, 1), dtype=np.int64)
    ln = np.zeros(max(n, 1), dtype=np.int64)
    lib().orc_plan_fixed_shards(D, shard_elems, _p(off, _i64p), _p(ln, _i64p))
    bucket = np.zeros(max(n, 1), dtype=np.int32)
    lib().orc_plan_buckets(_p(ln, _i64p), n, bucket_cap_elems, _p(bucket, _i32p))
    return ShardTable(off[:n], ln[:n], bucket[:n], D, offs[:len(numel)])


def plan_median(tensor_numel, bucket_cap_elems: int, interval: int, ref: int = 0,
                align: int = 4) -> ShardTable:
    """Sec. III-C: layers -> communication tensors (greedy, whole layers) ->
    median-based even slicing capped at the interval.  Every communication
    tensor starts at a multiple of `align` elements in the arena (each is a
    buffer of its own in the framework the paper builds on), layers inside it
    are tight; slices are multiples of `align` except the last of a tensor.
    The layout is worked out by orc_plan_median_layout; this only marshals."""
    numel = np.ascontiguousarray(tensor_numel, dtype=np.int64)
    n = len(numel)
    offs = np.zeros(max(n, 1), dtype=np.int64)
    arena = C.c_int64(0)
    count = lib().orc_plan_median_layout(_p(numel, _i64p), n, bucket_cap_elems, interval, ref, align,
                                         _p(offs, _i64p), None, None, None, C.byref(arena))
    off = np.zeros(max(count, 1), dtype=np.int64)
    ln = np.zeros(max(count, 1), dtype=np.int64)
    bucket = np.zeros(max(count, 1), dtype=np.int32)
    lib().orc_plan_median_layout(_p(numel, _i64p), n, bucket_cap_elems, interval, ref, align,
                                 _p(offs, _i64p), _p(off, _i64p), _p(ln, _i64p), _p(bucket, _i32p),
                                 C.byref(arena))
    return ShardTable(off[:count], ln[:count], bucket[:count], arena.value, offs[:n], align)


def median_parts(numel, ref: int, interval: int):
    numel = np.ascontiguousarray(numel, dtype=np.int64)
    parts = np.zeros(len(numel), dtype=np.int32)
    total = lib().orc_plan_median_parts(_p(numel, _i64p), len(numel), ref, interval,
                                        _p(parts, _i32p))
    return parts, int(total)


def even_slices(numel: int, parts: int, align: int):
    out = np.zeros(parts, dtype=np.int64)
    n = lib().orc_plan_even_slices(numel, parts, align, _p(out, _i64p))
    return out[:n]


def selected(s: int, t: int, interval: int) -> bool:
    return bool(lib().orc_selected(s, t, interval))


def _packed_end(tab: ShardTable, interval: int, t: int, sh_hi: int) -> int:
    return int(lib().orc_packed_end(_p(tab.len, _i64p), sh_hi, interval, t, tab.align))


def packed_base(tab: ShardTable, interval: int, t: int, bucket: int) -> int:
    """Where the bucket's first sent shard starts in the step's packed layout."""
    lo, _ = tab.bucket_range(bucket)
    a = tab.align
    return (_packed_end(tab, interval, t, lo) + a - 1) // a * a


def packed_elems(tab: ShardTable, interval: int, t: int, bucket: int = -1) -> int:
    """Extent of the packed range the bucket's sent shards occupy at step t
    (for the whole arena: the payload size), 0 if it sends nothing."""
    _, hi = tab.bucket_range(bucket)
    return max(0, _packed_end(tab, interval, t, hi) - packed_base(tab, interval, t, bucket))


# ------------------------------------------------------------------ hot path

def _kind(a: np.ndarray):
    if a.dtype == np.float32:
        return "f32", _f32p
    if a.dtype == np.uint16:
        return "bf16", _u16p
    raise TypeError("oracle arrays are float32, or uint16 holding bf16 bit patterns")


def compress(tab: ShardTable, interval: int, t: int, G, R, send, c: float = 1.0,
             bucket: int = -1, threads: int = 1) -> int:
    """In place: R becomes the new residual, send receives the packed shards.
    G/send uint16 (bf16 patterns) with R float32 selects the mixed-precision form;
    G/R float32 with send uint16 (fp16 patterns) the half-payload form.
    threads > 1: the same C routine is called on runs of whole shards from a thread pool."""
    lo, hi = tab.bucket_range(bucket)
    if G.dtype == np.float32 and send.dtype == np.uint16:
        _chk(G, np.float32), _chk(R, np.float32), _chk(send, np.uint16)
        f, args = lib().orc_compress_f32_pay16, (_p(G, _f32p), _p(R, _f32p), _p(send, _u16p))
    elif G.dtype == np.uint16 and R.dtype == np.float32:
        _chk(G, np.uint16), _chk(send, np.uint16), _chk(R, np.float32)
        f, args = lib().orc_compress_bf16_res32, (_p(G, _u16p), _p(R, _f32p), _p(send, _u16p))
    else:
        name, ptr = _kind(G)
        for a in (G, R, send):
            _chk(a, G.dtype)
        f, args = getattr(lib(), "orc_compress_" + name), (_p(G, ptr), _p(R, ptr), _p(send, ptr))
    off, ln = _p(tab.off, _i64p), _p(tab.len, _i64p)
    calls = [lambda a=a, b=b: f(*args, off, ln, a, b, interval, t, c, tab.align)
             for a, b in _ranges(tab, lo, hi, threads)]
    return int(sum(_run(calls, threads)))


def compress_aliased(tab: ShardTable, interval: int, t: int, accum, send, bucket: int = -1) -> int:
    """In place: sent shards of accum move to send and are cleared."""
    _chk(accum, accum.dtype), _chk(send, accum.dtype)
    lo, hi = tab.bucket_range(bucket)
    return int(lib().orc_compress_aliased(accum.ctypes.data, send.ctypes.data, accum.dtype.itemsize,
                                          _p(tab.off, _i64p), _p(tab.len, _i64p), lo, hi, interval, t,
                                          tab.align))


def decompress(tab: ShardTable, interval: int, t: int, recv, out, bucket: int = -1,
               threads: int = 1) -> None:
    """recv: [N, stride] packed payload rows; out: dense arena, fully written.
    recv uint16 with out float32 selects the half-payload form.
    threads > 1: the same C routine is called on runs of whole shards from a thread pool."""
    assert recv.ndim == 2
    lo, hi = tab.bucket_range(bucket)
    if recv.dtype == np.uint16 and out.dtype == np.float32:
        _chk(recv, np.uint16), _chk(out, np.float32)
        f, args = lib().orc_decompress_pay16, (_p(recv, _u16p), recv.shape[0], recv.shape[1], _p(out, _f32p))
    else:
        name, ptr = _kind(recv)
        _chk(recv, recv.dtype)
        _chk(out, recv.dtype)
        f = getattr(lib(), "orc_decompress_" + name)
        args = (_p(recv, ptr), recv.shape[0], recv.shape[1], _p(out, ptr))
    off, ln = _p(tab.off, _i64p), _p(tab.len, _i64p)
    calls = [lambda a=a, b=b: f(*args, off, ln, a, b, interval, t, tab.align)
             for a, b in _ranges(tab, lo, hi, threads)]
    _run(calls, threads)


def unpack_mean(tab: ShardTable, interval: int, t: int, summed, n_workers: int, out, bucket: int = -1,
                threads: int = 1) -> None:
    """The step after a sum-AllReduce: `summed` is one payload row (the element-wise sum of the
    workers' payloads), out = summed / n_workers where a shard was sent, +0 elsewhere.
    summed uint16 with out float32 selects the half-payload form."""
    lo, hi = tab.bucket_range(bucket)
    if summed.dtype == np.uint16 and out.dtype == np.float32:
        _chk(summed, np.uint16), _chk(out, np.float32)
        f, args = lib().orc_unpack_mean_pay16, (_p(summed, _u16p), n_workers, _p(out, _f32p))
    else:
        name, ptr = _kind(summed)
        _chk(summed, summed.dtype), _chk(out, summed.dtype)
        f, args = getattr(lib(), "orc_unpack_mean_" + name), (_p(summed, ptr), n_workers, _p(out, ptr))
    off, ln = _p(tab.off, _i64p), _p(tab.len, _i64p)
    calls = [lambda a=a, b=b: f(*args, off, ln, a, b, interval, t, tab.align)
             for a, b in _ranges(tab, lo, hi, threads)]
    _run(calls, threads)


def topk(G, R, k: int, c: float = 1.0):
    """In place on R.  Returns (vals[k] float32, idx[k] uint32) in ascending index."""
    _chk(G, np.float32)
    _chk(R, np.float32)
    vals = np.zeros(max(k, 1), dtype=np.float32)
    idx = np.zeros(max(k, 1), dtype=np.uint32)
    rc = lib().orc_topk_f32(_p(G, _f32p), _p(R, _f32p), G.shape[0], k, c, _p(vals, _f32p),
                            _p(idx, _u32p))
    if rc != 0:
        raise ValueError("orc_topk_f32: bad n or k")
    return vals[:k], idx[:k]


def randk(G, R, idx, c: float = 1.0):
    """In place on R.  idx: uint32, distinct.  Returns vals[k]."""
    _chk(G, np.float32), _chk(R, np.float32), _chk(idx, np.uint32)
    vals = np.zeros(max(len(idx), 1), np.float32)
    if lib().orc_randk_f32(_p(G, _f32p), _p(R, _f32p), G.shape[0], _p(idx, _u32p), len(idx), c,
                           _p(vals, _f32p)) != 0:
        raise ValueError("orc_randk_f32: bad n or k")
    return vals[:len(idx)]


def fp16_compress(G, R, c: float = 1.0):
    """In place on R.  Returns the fp16 payload as uint16 bit patterns."""
    _chk(G, np.float32), _chk(R, np.float32)
    out = np.zeros(G.shape[0], np.uint16)
    lib().orc_fp16_compress(_p(G, _f32p), _p(R, _f32p), G.shape[0], c, _p(out, _u16p))
    return out


def fp16_mean(recv, n: int):
    _chk(recv, np.uint16)
    out = np.zeros(n, np.float32)
    lib().orc_fp16_mean(_p(recv, _u16p), recv.shape[0], recv.shape[1], n, _p(out, _f32p))
    return out


def sparse_mean(vals, idx, k: int, n: int):
    _chk(vals, np.float32), _chk(idx, np.uint32)
    out = np.zeros(n, np.float32)
    lib().orc_sparse_mean(_p(vals, _f32p), _p(idx, _u32p), vals.shape[0], k, vals.shape[1], n,
                          _p(out, _f32p))
    return out


def f32_to_f16(x: float) -> int:
    return int(lib().orc_f32_to_f16(x))


def f16_to_f32(h: int) -> float:
    return float(lib().orc_f16_to_f32(h))


def f32_to_bf16(x: float) -> int:
    return int(lib().orc_f32_to_bf16(x))


def bf16_to_f32(h: int) -> float:
    return float(lib().orc_bf16_to_f32(h))


# ------------------------------------------------------------------ policy

def ratio_from_ccr(ccr: float) -> int:
    k = C.c_int32(0)
    if lib().orc_ratio_from_ccr(ccr, C.byref(k)) != 0:
        raise ValueError("CCR must be a positive finite number")
    return int(k.value)


def ef_coeff(init_value: float, num_steps: int, ascend_steps: int, ascend_range: float) -> float:
    if ascend_steps <= 0:
        raise ValueError("ascend_steps must be positive")
    return float(lib().orc_ef_coeff(init_value, num_steps, ascend_steps, ascend_range))
