"""Thin ctypes binding over libcovap.so (the C ABI declared in include/covap.h).

Argument marshalling only: every step of the hot path runs in the library's
HIP kernels.  torch is used for device memory and streams; tensors are passed
as raw device pointers.  There is no fallback: if the library is not built (or
cannot be loaded) the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_CSRC = os.path.join(_HERE, "csrc")
_INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_HERE, "libcovap.so")

SOURCES = ["plan.cpp", "kernels.hip", "topk.hip", "contrast.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # the only FMA is the one written as fmaf
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unknown-attributes",
]

COVAP_F32, COVAP_BF16, COVAP_BF16_RES32, COVAP_F32_PAY16 = 0, 1, 2, 3
COVAP_SHARD_FIXED, COVAP_SHARD_MEDIAN = 0, 1
STATUS_NAMES = {0: "COVAP_OK", 1: "COVAP_EINVAL", 2: "COVAP_ENOMEM", 3: "COVAP_EHIP",
                4: "COVAP_ERANGE", 5: "COVAP_EUNSUPPORTED"}


class CovapError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


def build(verbose: bool = False) -> str:
    """Compile libcovap.so for gfx950 with hipcc (cross-compiles without a GPU)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(_CSRC, s) for s in SOURCES if os.path.exists(os.path.join(_CSRC, s))]
    cmd = [hipcc, *HIPCC_FLAGS, "-I", _INCLUDE, "-I", _CSRC, "-o", LIB_PATH, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB_PATH


class _PlanOpts(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("mode", C.c_int32), ("shard_elems", C.c_int64),
                ("bucket_cap_bytes", C.c_int64), ("ref_elems", C.c_int64), ("K", C.c_int32),
                ("reserved", C.c_int32)]


_lib = None
_vp = C.c_void_p
_i64p = C.POINTER(C.c_int64)
_i32p = C.POINTER(C.c_int32)


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                           "g.build()'` first (there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    L.covap_plan.restype = C.c_int
    L.covap_plan.argtypes = [_i64p, C.c_int32, C.POINTER(_PlanOpts), C.POINTER(_vp)]
    L.covap_plan_free.restype = None
    L.covap_plan_free.argtypes = [_vp]
    for name in ("covap_plan_total_elems", "covap_plan_packed_elems_max"):
        getattr(L, name).restype = C.c_int64
        getattr(L, name).argtypes = [_vp]
    for name in ("covap_plan_num_tensors", "covap_plan_num_shards", "covap_plan_num_buckets",
                 "covap_plan_interval", "covap_plan_align_elems"):
        getattr(L, name).restype = C.c_int32
        getattr(L, name).argtypes = [_vp]
    L.covap_plan_tensor_offset.restype = C.c_int64
    L.covap_plan_tensor_offset.argtypes = [_vp, C.c_int32]
    L.covap_plan_shard.restype = C.c_int
    L.covap_plan_shard.argtypes = [_vp, C.c_int32, _i64p, _i64p, _i32p]
    L.covap_plan_bucket.restype = C.c_int
    L.covap_plan_bucket.argtypes = [_vp, C.c_int32, _i32p, _i32p]
    L.covap_plan_is_selected.restype = C.c_int32
    L.covap_plan_is_selected.argtypes = [_vp, C.c_uint64, C.c_int32]
    L.covap_plan_selected.restype = C.c_int32
    L.covap_plan_selected.argtypes = [_vp, C.c_uint64, _i32p, C.c_int32]
    L.covap_plan_packed_elems.restype = C.c_int64
    L.covap_plan_packed_elems.argtypes = [_vp, C.c_uint64, C.c_int32]
    L.covap_plan_packed_base.restype = C.c_int64
    L.covap_plan_packed_base.argtypes = [_vp, C.c_uint64, C.c_int32]
    L.covap_plan_trace.restype = C.c_int64
    L.covap_plan_trace.argtypes = [_vp, C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.c_int64, _vp, _vp, _vp, _vp,
                                   _i32p, _i64p]
    L.covap_ratio_from_ccr.restype = C.c_int
    L.covap_ratio_from_ccr.argtypes = [C.c_double, _i32p]
    L.covap_ratio_from_times.restype = C.c_int
    L.covap_ratio_from_times.argtypes = [C.c_double, C.c_double, _i32p]
    L.covap_ef_coeff.restype = C.c_int
    L.covap_ef_coeff.argtypes = [C.c_float, C.c_uint64, C.c_uint64, C.c_float, C.POINTER(C.c_float)]
    L.covap_compress.restype = C.c_int
    L.covap_compress.argtypes = [_vp, C.c_uint64, C.c_int32, _vp, _vp, _vp, C.c_int64, C.c_float, _vp]
    L.covap_compress_bounded.restype = C.c_int
    L.covap_compress_bounded.argtypes = [_vp, C.c_uint64, C.c_int32, _vp, _vp, _vp, C.c_int64, C.c_float, C.c_int32,
                                         _vp]
    L.covap_compress_aliased.restype = C.c_int
    L.covap_compress_aliased.argtypes = [_vp, C.c_uint64, C.c_int32, _vp, _vp, C.c_int64, _vp]
    L.covap_decompress.restype = C.c_int
    L.covap_decompress.argtypes = [_vp, C.c_uint64, C.c_int32, _vp, C.c_int32, C.c_int64, _vp, _vp]
    L.covap_decompress_reduced.restype = C.c_int
    L.covap_decompress_reduced.argtypes = [_vp, C.c_uint64, C.c_int32, _vp, C.c_int32, _vp, _vp]
    L.topk_workspace_bytes.restype = C.c_size_t
    L.topk_workspace_bytes.argtypes = [C.c_int64, C.c_int32]
    L.topk_compress.restype = C.c_int
    L.topk_compress.argtypes = [_vp, _vp, C.c_int64, C.c_int64, C.c_int32, C.c_float, _vp, _vp, _vp,
                                C.c_size_t, _vp]
    L.topk_static_max_elems.restype = C.c_int64
    L.topk_static_max_elems.argtypes = []
    L.topk_compress_static.restype = C.c_int
    L.topk_compress_static.argtypes = [_vp, _vp, C.c_int64, C.c_int64, C.c_int32, C.c_float, _vp, _vp, _vp]
    L.randk_compress.restype = C.c_int
    L.randk_compress.argtypes = [_vp, _vp, C.c_int64, _vp, C.c_int64, C.c_float, _vp, _vp]
    L.fp16_compress.restype = C.c_int
    L.fp16_compress.argtypes = [_vp, _vp, C.c_int64, C.c_float, _vp, _vp]
    L.fp16_decompress.restype = C.c_int
    L.fp16_decompress.argtypes = [_vp, C.c_int32, C.c_int64, C.c_int64, _vp, _vp]
    L.sparse_decompress.restype = C.c_int
    L.sparse_decompress.argtypes = [_vp, _vp, C.c_int32, C.c_int64, C.c_int64, C.c_int64, _vp, _vp]
    L.sparse_decompress_sorted.restype = C.c_int
    L.sparse_decompress_sorted.argtypes = [_vp, _vp, C.c_int32, C.c_int64, C.c_int64, C.c_int64, _vp, _vp]
    L.covap_probe_copy.restype = C.c_int
    L.covap_probe_copy.argtypes = [_vp, _vp, C.c_size_t, _vp]
    L.covap_probe_triad.restype = C.c_int
    L.covap_probe_triad.argtypes = [_vp, _vp, _vp, C.c_float, C.c_int64, _vp]
    L.covap_probe_mfma.restype = C.c_int
    L.covap_probe_mfma.argtypes = [_vp, C.c_int32, C.c_int32, C.c_int32, _vp]
    L.covap_tune_set.restype = C.c_int
    L.covap_tune_set.argtypes = [C.c_char_p, C.c_int32]
    L.covap_tune_get.restype = C.c_int32
    L.covap_tune_get.argtypes = [C.c_char_p]
    L.covap_last_error.restype = C.c_char_p
    L.covap_last_error.argtypes = []
    L.covap_version.restype = C.c_char_p
    L.covap_version.argtypes = []
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        raise CovapError(status, lib().covap_last_error().decode())


def _ptr(t) -> int:
    """Device (or host) address of a torch tensor / numpy array / int."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        if not t.is_contiguous():
            raise ValueError("tensor must be contiguous")
        return t.data_ptr()
    return t.ctypes.data


def _need(t, what: str, elems: int, esz: Optional[int] = None) -> None:
    """The kernels trust the sizes they are given, and a read or write past an allocation
    is a GPU memory fault: refuse a tensor (or array) that is too small or of the wrong
    element width before its address is taken.  Raw integer addresses are the caller's
    responsibility."""
    if t is None or isinstance(t, int):
        return
    n = t.numel() if hasattr(t, "numel") else t.size
    if n < elems:
        raise ValueError(f"{what}: {n} elements, the call needs at least {elems}")
    if esz is not None:
        w = t.element_size() if hasattr(t, "element_size") else t.itemsize
        if w != esz:
            raise ValueError(f"{what}: {w}-byte elements, the plan's element type has {esz}")


_GRAD_ESZ = {COVAP_F32: 4, COVAP_BF16: 2, COVAP_BF16_RES32: 2, COVAP_F32_PAY16: 4}
_RESIDUAL_ESZ = {COVAP_F32: 4, COVAP_BF16: 2, COVAP_BF16_RES32: 4, COVAP_F32_PAY16: 4}
_PAYLOAD_ESZ = {COVAP_F32: 4, COVAP_BF16: 2, COVAP_BF16_RES32: 2, COVAP_F32_PAY16: 2}


def _stream(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Plan:
    """Owner of a covap_plan_t handle."""

    def __init__(self, handle: int, dtype: int):
        self._h = handle
        self.dtype = dtype

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:          # at interpreter exit the module may be gone already
            _lib.covap_plan_free(h)

    @property
    def handle(self) -> int:
        return self._h

    total_elems = property(lambda self: lib().covap_plan_total_elems(self._h))
    num_tensors = property(lambda self: lib().covap_plan_num_tensors(self._h))
    num_shards = property(lambda self: lib().covap_plan_num_shards(self._h))
    num_buckets = property(lambda self: lib().covap_plan_num_buckets(self._h))
    interval = property(lambda self: lib().covap_plan_interval(self._h))
    align_elems = property(lambda self: lib().covap_plan_align_elems(self._h))
    packed_elems_max = property(lambda self: lib().covap_plan_packed_elems_max(self._h))

    def tensor_offset(self, i: int) -> int:
        return lib().covap_plan_tensor_offset(self._h, i)

    def shard(self, s: int):
        off, ln, b = C.c_int64(), C.c_int64(), C.c_int32()
        _check(lib().covap_plan_shard(self._h, s, C.byref(off), C.byref(ln), C.byref(b)))
        return off.value, ln.value, b.value

    def bucket(self, b: int):
        lo, hi = C.c_int32(), C.c_int32()
        _check(lib().covap_plan_bucket(self._h, b, C.byref(lo), C.byref(hi)))
        return lo.value, hi.value

    def is_selected(self, step: int, s: int) -> int:
        return lib().covap_plan_is_selected(self._h, step, s)

    def selected(self, step: int):
        n = lib().covap_plan_selected(self._h, step, None, 0)
        ids = (C.c_int32 * max(n, 1))()
        lib().covap_plan_selected(self._h, step, ids, n)
        return list(ids[:n])

    def packed_elems(self, step: int, bucket: int = -1) -> int:
        return lib().covap_plan_packed_elems(self._h, step, bucket)

    def packed_base(self, step: int, bucket: int = -1) -> int:
        return lib().covap_plan_packed_base(self._h, step, bucket)

    def trace(self, step: int, bucket: int = -1, tile_elems: int = 256, sent_only: bool = False):
        """Host replay of the call's launches: numpy arrays (off, poff, n, sel) of the
        tiles in launch order, plus (launches, workgroups)."""
        import numpy as np
        nl, nw = C.c_int32(), C.c_int64()
        cnt = lib().covap_plan_trace(self._h, step, bucket, tile_elems, int(sent_only), 0, None, None, None,
                                     None, C.byref(nl), C.byref(nw))
        if cnt < 0:
            raise CovapError(1, lib().covap_last_error().decode())
        off, poff = np.empty(cnt, np.int64), np.empty(cnt, np.int64)
        n, sel = np.empty(cnt, np.int32), np.empty(cnt, np.uint8)
        lib().covap_plan_trace(self._h, step, bucket, tile_elems, int(sent_only), cnt, off.ctypes.data,
                               poff.ctypes.data, n.ctypes.data, sel.ctypes.data, None, None)
        return off, poff, n, sel, nl.value, nw.value


def covap_plan(tensor_numel: Sequence[int], shard_elems: int, K: int, dtype: int = COVAP_F32,
               bucket_cap_bytes: int = 25 << 20, mode: int = COVAP_SHARD_FIXED,
               ref_elems: int = 0) -> Plan:
    arr = (C.c_int64 * max(len(tensor_numel), 1))(*[int(x) for x in tensor_numel])
    opts = _PlanOpts(dtype, mode, shard_elems, bucket_cap_bytes, ref_elems, K, 0)
    h = _vp()
    _check(lib().covap_plan(arr, len(tensor_numel), C.byref(opts), C.byref(h)))
    return Plan(h.value, dtype)


def covap_compress(plan: Plan, step: int, grad, residual, send, ef_coeff: float = 1.0,
                   bucket: int = -1, stream=None, send_cap_elems: Optional[int] = None,
                   max_workgroups: Optional[int] = None) -> None:
    """covap_compress, or covap_compress_bounded when max_workgroups is given."""
    cap = send.numel() if send_cap_elems is None else send_cap_elems
    D = plan.total_elems                      # with median sharding this includes alignment padding
    _need(grad, "grad", D, _GRAD_ESZ[plan.dtype])
    _need(residual, "residual", D, _RESIDUAL_ESZ[plan.dtype])
    _need(send, "send", cap, _PAYLOAD_ESZ[plan.dtype])
    if max_workgroups is None:
        _check(lib().covap_compress(plan.handle, step, bucket, _ptr(grad), _ptr(residual), _ptr(send),
                                    cap, ef_coeff, _stream(stream)))
    else:
        _check(lib().covap_compress_bounded(plan.handle, step, bucket, _ptr(grad), _ptr(residual),
                                            _ptr(send), cap, ef_coeff, max_workgroups, _stream(stream)))


def covap_compress_aliased(plan: Plan, step: int, accum, send, bucket: int = -1, stream=None,
                           send_cap_elems: Optional[int] = None) -> None:
    cap = send.numel() if send_cap_elems is None else send_cap_elems
    _need(accum, "accum", plan.total_elems, _GRAD_ESZ[plan.dtype])
    _need(send, "send", cap, _PAYLOAD_ESZ[plan.dtype])
    _check(lib().covap_compress_aliased(plan.handle, step, bucket, _ptr(accum), _ptr(send), cap,
                                        _stream(stream)))


def covap_decompress(plan: Plan, step: int, recv, dense_out, n_workers: Optional[int] = None,
                     stride_elems: Optional[int] = None, bucket: int = -1, stream=None) -> None:
    if n_workers is None:
        n_workers = recv.shape[0]
    if stride_elems is None:
        stride_elems = recv.stride(0) if recv.dim() == 2 else recv.numel()
    used = plan.packed_elems(step, bucket)
    if used > 0 and n_workers >= 1:
        _need(recv, "recv", (n_workers - 1) * stride_elems + plan.packed_base(step, bucket) + used,
              _PAYLOAD_ESZ[plan.dtype])
    _need(dense_out, "dense_out", plan.total_elems, _GRAD_ESZ[plan.dtype])
    _check(lib().covap_decompress(plan.handle, step, bucket, _ptr(recv), n_workers, stride_elems,
                                  _ptr(dense_out), _stream(stream)))


def covap_decompress_reduced(plan: Plan, step: int, summed, dense_out, n_workers: int, bucket: int = -1,
                             stream=None) -> None:
    used = plan.packed_elems(step, bucket)
    if used > 0:
        _need(summed, "summed", plan.packed_base(step, bucket) + used, _PAYLOAD_ESZ[plan.dtype])
    _need(dense_out, "dense_out", plan.total_elems, _GRAD_ESZ[plan.dtype])
    _check(lib().covap_decompress_reduced(plan.handle, step, bucket, _ptr(summed), n_workers, _ptr(dense_out),
                                          _stream(stream)))


def topk_workspace_bytes(n: int, dtype: int = COVAP_F32) -> int:
    return lib().topk_workspace_bytes(n, dtype)


def topk_compress(grad, residual, k: int, out_vals, out_idx, workspace, ef_coeff: float = 1.0,
                  n: Optional[int] = None, dtype: int = COVAP_F32, stream=None,
                  ws_bytes: Optional[int] = None) -> None:
    if n is None:
        n = grad.numel()
    if ws_bytes is None:
        ws_bytes = workspace.numel() * workspace.element_size()
    _need(grad, "grad", n, 4), _need(residual, "residual", n, 4)
    _need(out_vals, "out_vals", k, 4), _need(out_idx, "out_idx", k, 4)
    if not isinstance(workspace, int) and workspace is not None:
        _need(workspace, "workspace", -(-ws_bytes // workspace.element_size()))
    _check(lib().topk_compress(_ptr(grad), _ptr(residual), n, k, dtype, ef_coeff, _ptr(out_vals),
                               _ptr(out_idx), _ptr(workspace), ws_bytes, _stream(stream)))


def topk_static_max_elems() -> int:
    return lib().topk_static_max_elems()


def topk_compress_static(grad, residual, k: int, out_vals, out_idx, ef_coeff: float = 1.0,
                         n: Optional[int] = None, dtype: int = COVAP_F32, stream=None) -> None:
    """topk_compress on the library's built-in workspace (no allocation anywhere)."""
    if n is None:
        n = grad.numel()
    _need(grad, "grad", n, 4), _need(residual, "residual", n, 4)
    _need(out_vals, "out_vals", k, 4), _need(out_idx, "out_idx", k, 4)
    _check(lib().topk_compress_static(_ptr(grad), _ptr(residual), n, k, dtype, ef_coeff,
                                      _ptr(out_vals), _ptr(out_idx), _stream(stream)))


def randk_compress(grad, residual, idx, out_vals, ef_coeff: float = 1.0, n: Optional[int] = None,
                   k: Optional[int] = None, stream=None) -> None:
    n = grad.numel() if n is None else n
    k = idx.numel() if k is None else k
    _need(grad, "grad", n, 4), _need(residual, "residual", n, 4)
    _need(idx, "idx", k, 4), _need(out_vals, "out_vals", k, 4)
    _check(lib().randk_compress(_ptr(grad), _ptr(residual), n, _ptr(idx), k, ef_coeff,
                                _ptr(out_vals), _stream(stream)))


def fp16_compress(grad, residual, out_half, ef_coeff: float = 1.0, n: Optional[int] = None,
                  stream=None) -> None:
    n = grad.numel() if n is None else n
    _need(grad, "grad", n, 4), _need(residual, "residual", n, 4), _need(out_half, "out_half", n, 2)
    _check(lib().fp16_compress(_ptr(grad), _ptr(residual), n, ef_coeff, _ptr(out_half), _stream(stream)))


def fp16_decompress(recv, dense_out, n: Optional[int] = None, n_workers: Optional[int] = None,
                    stride_elems: Optional[int] = None, stream=None) -> None:
    n_workers = recv.shape[0] if n_workers is None else n_workers
    stride_elems = recv.stride(0) if stride_elems is None else stride_elems
    n = dense_out.numel() if n is None else n
    if n_workers >= 1:
        _need(recv, "recv", (n_workers - 1) * stride_elems + n, 2)
    _need(dense_out, "dense_out", n, 4)
    _check(lib().fp16_decompress(_ptr(recv), n_workers, stride_elems, n, _ptr(dense_out), _stream(stream)))


def sparse_decompress(vals, idx, dense_out, k: Optional[int] = None, n: Optional[int] = None,
                      n_workers: Optional[int] = None, stride_elems: Optional[int] = None,
                      stream=None) -> None:
    n_workers = vals.shape[0] if n_workers is None else n_workers
    stride_elems = vals.stride(0) if stride_elems is None else stride_elems
    k = vals.shape[1] if k is None else k
    n = dense_out.numel() if n is None else n
    if n_workers >= 1 and k > 0:
        _need(vals, "vals", (n_workers - 1) * stride_elems + k, 4)
        _need(idx, "idx", (n_workers - 1) * stride_elems + k, 4)
    _need(dense_out, "dense_out", n, 4)
    _check(lib().sparse_decompress(_ptr(vals), _ptr(idx), n_workers, k, stride_elems, n,
                                   _ptr(dense_out), _stream(stream)))


def sparse_decompress_sorted(vals, idx, dense_out, k: Optional[int] = None, n: Optional[int] = None,
                             n_workers: Optional[int] = None, stride_elems: Optional[int] = None,
                             stream=None) -> None:
    n_workers = vals.shape[0] if n_workers is None else n_workers
    stride_elems = vals.stride(0) if stride_elems is None else stride_elems
    k = vals.shape[1] if k is None else k
    n = dense_out.numel() if n is None else n
    if n_workers >= 1 and k > 0:
        _need(vals, "vals", (n_workers - 1) * stride_elems + k, 4)
        _need(idx, "idx", (n_workers - 1) * stride_elems + k, 4)
    _need(dense_out, "dense_out", n, 4)
    _check(lib().sparse_decompress_sorted(_ptr(vals), _ptr(idx), n_workers, k, stride_elems, n,
                                          _ptr(dense_out), _stream(stream)))


def covap_ratio_from_ccr(ccr: float) -> int:
    k = C.c_int32()
    _check(lib().covap_ratio_from_ccr(ccr, C.byref(k)))
    return k.value


def covap_ratio_from_times(t_comm: float, t_comp: float) -> int:
    k = C.c_int32()
    _check(lib().covap_ratio_from_times(t_comm, t_comp, C.byref(k)))
    return k.value


def covap_ef_coeff(init_value: float, num_steps: int, ascend_steps: int, ascend_range: float) -> float:
    c = C.c_float()
    _check(lib().covap_ef_coeff(init_value, num_steps, ascend_steps, ascend_range, C.byref(c)))
    return c.value


def covap_probe_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(lib().covap_probe_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


def covap_probe_triad(a, b, c, s: float, n: int, stream=None) -> None:
    _check(lib().covap_probe_triad(_ptr(a), _ptr(b), _ptr(c), s, n, _stream(stream)))


def covap_probe_mfma(out, workgroups: int, iters: int, lds_bytes: int = 0, stream=None) -> None:
    _need(out, "out", workgroups * 256, 4)
    _check(lib().covap_probe_mfma(_ptr(out), workgroups, iters, lds_bytes, _stream(stream)))


def covap_tune_set(key: str, value: int) -> None:
    _check(lib().covap_tune_set(key.encode(), value))


def covap_tune_get(key: str) -> int:
    return lib().covap_tune_get(key.encode())


def covap_version() -> str:
    return lib().covap_version().decode()
