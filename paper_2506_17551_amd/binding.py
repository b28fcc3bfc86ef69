"""ctypes binding of libgradcomp.so: same names as the C ABI (include/gradcomp.h),
argument marshalling only. Every step of the path runs in the library's kernels;
if the library is missing or fails to load this module raises — there is no
fallback implementation."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

from . import build as _build

GC_OK, GC_ERR_INVALID_ARG, GC_ERR_UNSUPPORTED, GC_ERR_WORKSPACE, GC_ERR_NONFINITE, GC_ERR_DEVICE = range(6)
GC_F32, GC_BF16 = 0, 1
GC_CODEC_INT8, GC_CODEC_SIGN1 = 0, 1


class GradCompError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_status_string(status)} (gc_status {status})")


class _GcBuf(ctypes.Structure):
    _fields_ = [("indices", ctypes.c_void_p), ("q", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("n", ctypes.c_int64), ("k", ctypes.c_int64), ("block", ctypes.c_int32),
                ("index_bits", ctypes.c_int32), ("codec", ctypes.c_int32), ("reserved_", ctypes.c_int32)]


class _GcStats(ctypes.Structure):
    _fields_ = [("tensors", ctypes.c_int64), ("tensors_sampled", ctypes.c_int64),
                ("tensors_fallback", ctypes.c_int64), ("candidates", ctypes.c_int64)]


EXPORTS = ["gc_create", "gc_destroy", "gc_reserve", "gc_k_from_density", "gc_num_scales", "gc_num_code_bytes", "gc_compress",
           "gc_compress_multi", "gc_decompress_sum", "gc_decompress_sum_static", "gc_decompress_sum_multi", "gc_decompress_sum_weighted",
           "gc_decompress_apply", "gc_compress_rows", "gc_decompress_sum_rows", "gc_compress_dense", "gc_decompress_sum_dense", "gc_decompress_apply_dense",
           "gc_sync_status",
           "gc_last_stats", "gc_profile_enable", "gc_profile_num_kernels", "gc_profile_kernel_name",
           "gc_profile_read", "gc_set_option", "gc_status_string"]

_lib = None


def lib() -> ctypes.CDLL:
    """Load libgradcomp.so (building it once if it has never been built). Raises if that fails."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.ensure_library()
    L = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    L.gc_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    L.gc_destroy.argtypes = [vp]
    L.gc_reserve.argtypes = [vp, i64, i64, i32, i32]
    L.gc_k_from_density.argtypes = [i64, ctypes.c_double]
    L.gc_k_from_density.restype = i64
    L.gc_num_scales.argtypes = [i64, i32]
    L.gc_num_scales.restype = i64
    L.gc_num_code_bytes.argtypes = [i64, i32, ctypes.c_int]
    L.gc_num_code_bytes.restype = i64
    L.gc_compress.argtypes = [vp, vp, ctypes.c_int, vp, i64, i64, i32, ctypes.POINTER(_GcBuf), vp]
    L.gc_compress_multi.argtypes = [vp, vp, ctypes.c_int, vp, vp, vp, i32, i32, ctypes.POINTER(_GcBuf), vp]
    L.gc_decompress_sum.argtypes = [vp, ctypes.POINTER(_GcBuf), i32, vp, i64, vp]
    L.gc_decompress_sum_static.argtypes = [vp, ctypes.POINTER(_GcBuf), i32, vp, i64, vp]
    L.gc_decompress_sum_multi.argtypes = [vp, ctypes.POINTER(_GcBuf), i32, vp, i32, vp, i64, vp]
    L.gc_decompress_sum_weighted.argtypes = [vp, ctypes.POINTER(_GcBuf), i32, vp, i32, vp, vp, i64, vp]
    L.gc_decompress_apply.argtypes = [vp, ctypes.POINTER(_GcBuf), i32, vp, i32, vp, vp, ctypes.c_float, i64, vp]
    L.gc_compress_rows.argtypes = [vp, vp, ctypes.c_int, vp, vp, i64, i64, i64, i64, i32, ctypes.POINTER(_GcBuf), vp]
    L.gc_decompress_sum_rows.argtypes = [vp, ctypes.POINTER(_GcBuf), i32, vp, i64, i64, vp, vp, vp]
    L.gc_compress_dense.argtypes = [vp, vp, ctypes.c_int, vp, i64, i32, ctypes.c_int, vp, vp, vp]
    L.gc_decompress_sum_dense.argtypes = [vp, vp, vp, i32, i32, ctypes.c_int, vp, vp, i64, vp]
    L.gc_decompress_apply_dense.argtypes = [vp, vp, vp, i32, i32, ctypes.c_int, vp, vp, ctypes.c_float, i64, vp]
    L.gc_sync_status.argtypes = [vp, vp]
    L.gc_last_stats.argtypes = [vp, ctypes.POINTER(_GcStats)]
    L.gc_profile_enable.argtypes = [vp, i32]
    L.gc_profile_num_kernels.restype = i32
    L.gc_profile_kernel_name.argtypes = [i32]
    L.gc_profile_kernel_name.restype = ctypes.c_char_p
    L.gc_profile_read.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    L.gc_set_option.argtypes = [vp, ctypes.c_char_p, i64]
    L.gc_set_option.restype = ctypes.c_int
    L.gc_status_string.argtypes = [ctypes.c_int]
    L.gc_status_string.restype = ctypes.c_char_p
    for name in ("gc_create", "gc_destroy", "gc_reserve", "gc_compress", "gc_compress_multi", "gc_decompress_sum",
                 "gc_decompress_sum_static",
                 "gc_decompress_sum_multi", "gc_decompress_sum_weighted", "gc_decompress_apply",
                 "gc_compress_rows", "gc_decompress_sum_rows", "gc_compress_dense", "gc_decompress_sum_dense", "gc_decompress_apply_dense",
                 "gc_sync_status", "gc_last_stats", "gc_profile_enable",
                 "gc_profile_read"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def _status_string(s: int) -> str:
    return lib().gc_status_string(int(s)).decode()


def _check(status: int, where: str) -> None:
    if status != GC_OK:
        raise GradCompError(status, where)


def k_from_density(n: int, density: float) -> int:
    return int(lib().gc_k_from_density(int(n), float(density)))


def num_scales(k: int, block: int) -> int:
    return int(lib().gc_num_scales(int(k), int(block)))


def num_code_bytes(k: int, block: int, codec: int = GC_CODEC_INT8) -> int:
    return int(lib().gc_num_code_bytes(int(k), int(block), int(codec)))


def _stream_ptr(stream: Optional[torch.cuda.Stream], device) -> int:
    s = stream if stream is not None else torch.cuda.current_stream(device)
    return int(s.cuda_stream)


class Context:
    """Owns the library's scratch workspace on one device (gc_ctx)."""

    def __init__(self, device: int = 0):
        self.device = int(device)
        h = ctypes.c_void_p()
        _check(lib().gc_create(ctypes.byref(h), self.device), "gc_create")
        self._h = h

    @property
    def handle(self) -> ctypes.c_void_p:
        if self._h is None:
            raise RuntimeError("context destroyed")
        return self._h

    def destroy(self) -> None:
        if self._h is not None:
            lib().gc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def reserve(self, max_n: int, max_k: int, max_tensors: int = 1, max_W: int = 0) -> None:
        """gc_reserve: size the workspace once; later calls within these bounds never allocate."""
        _check(lib().gc_reserve(self.handle, int(max_n), int(max_k), int(max_tensors), int(max_W)), "gc_reserve")

    def set_option(self, name: str, value: int) -> None:
        _check(lib().gc_set_option(self.handle, name.encode(), int(value)), "gc_set_option")

    # ---- profiling helpers (gc_profile_*) ----
    def profile_enable(self, mode=1) -> None:
        """0/False: off, 1/True: every kernel, 2: only the streaming pass of compress."""
        _check(lib().gc_profile_enable(self.handle, int(mode)), "gc_profile_enable")

    def profile_read(self) -> dict:
        """{kernel name: (total ms, launches)} since profile_enable(True)."""
        out = {}
        L = lib()
        for i in range(L.gc_profile_num_kernels()):
            ms, cnt = ctypes.c_double(), ctypes.c_int64()
            _check(L.gc_profile_read(self.handle, i, ctypes.byref(ms), ctypes.byref(cnt)), "gc_profile_read")
            out[L.gc_profile_kernel_name(i).decode()] = (ms.value, cnt.value)
        return out


@dataclass
class CompressedBuf:
    """Device tensors of one compressed gradient (a gc_buf). `indices` holds unsigned values in a
    signed torch dtype of the same width (int32 for 32-bit, int64 for 64-bit indices)."""
    indices: torch.Tensor
    q: torch.Tensor
    scales: torch.Tensor
    n: int
    k: int
    block: int
    index_bits: int
    codec: int = GC_CODEC_INT8

    def struct(self) -> _GcBuf:
        return _GcBuf(self.indices.data_ptr(), self.q.data_ptr(), self.scales.data_ptr(), self.n, self.k,
                      self.block, self.index_bits, self.codec, 0)

    def indices_numpy(self) -> np.ndarray:
        a = self.indices.detach().cpu().numpy()
        return a.view(np.uint32) if self.index_bits == 32 else a.view(np.uint64)

    @staticmethod
    def allocate(n: int, k: int, nscales: int, block: int, index_bits: int, device, codec: int = GC_CODEC_INT8,
                 code_bytes: Optional[int] = None) -> "CompressedBuf":
        it = torch.int32 if index_bits == 32 else torch.int64
        nq = k if codec == GC_CODEC_INT8 else (code_bytes if code_bytes is not None
                                               else num_code_bytes(k, max(block, 1), codec))
        return CompressedBuf(torch.empty(k, dtype=it, device=device),
                             torch.empty(max(nq, 1), dtype=torch.int8, device=device)[:nq],
                             torch.empty(max(nscales, 1), dtype=torch.float32, device=device)[:nscales],
                             int(n), int(k), int(block), int(index_bits), int(codec))


def _grad_dtype(grad: torch.Tensor) -> int:
    if grad.dtype == torch.float32:
        return GC_F32
    if grad.dtype == torch.bfloat16:
        return GC_BF16
    raise TypeError("grad must be float32 or bfloat16")


def _check_dev(t: torch.Tensor, name: str, dtype=None) -> None:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}")


def compress(ctx: Context, grad: torch.Tensor, residual: torch.Tensor, k: int, block: int,
             out: Optional[CompressedBuf] = None, index_bits: Optional[int] = None,
             stream: Optional[torch.cuda.Stream] = None, codec: int = GC_CODEC_INT8) -> CompressedBuf:
    """gc_compress: one error-feedback step on one flat tensor; `residual` is updated in place."""
    _check_dev(grad, "grad")
    _check_dev(residual, "residual", torch.float32)
    n = grad.numel()
    if residual.numel() != n:
        raise ValueError("grad and residual differ in length")
    if index_bits is None:
        index_bits = 64 if n > (1 << 32) else 32
    if out is None:
        kk = max(int(k), 0)
        out = CompressedBuf.allocate(n, kk, num_scales(kk, block), block, index_bits, grad.device, codec)
    st = out.struct()
    rc = lib().gc_compress(ctx.handle, grad.data_ptr(), _grad_dtype(grad), residual.data_ptr(), n, int(k),
                           int(block), ctypes.byref(st), _stream_ptr(stream, grad.device))
    _check(rc, "gc_compress")
    return out


def compress_multi(ctx: Context, grad: torch.Tensor, residual: torch.Tensor, offsets: Sequence[int],
                   ks: Sequence[int], block: int, out: Optional[CompressedBuf] = None,
                   index_bits: Optional[int] = None,
                   stream: Optional[torch.cuda.Stream] = None, codec: int = GC_CODEC_INT8) -> CompressedBuf:
    """gc_compress_multi: per-tensor top-k over tensors stored back to back in one flat buffer."""
    _check_dev(grad, "grad")
    _check_dev(residual, "residual", torch.float32)
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    kk = np.ascontiguousarray(ks, dtype=np.int64)
    T = kk.shape[0]
    if off.shape[0] != T + 1:
        raise ValueError("offsets must have len(ks) + 1 entries")
    n = grad.numel()
    if residual.numel() != n:
        raise ValueError("grad and residual differ in length")
    if index_bits is None:
        index_bits = 64 if n > (1 << 32) else 32
    if out is None:
        ktot = int(kk.clip(min=0).sum())
        stot = int(sum(num_scales(int(x), block) for x in kk))
        qtot = int(sum(num_code_bytes(int(x), block, codec) for x in kk)) if block > 0 else 0
        out = CompressedBuf.allocate(n, ktot, stot, block, index_bits, grad.device, codec, qtot)
    st = out.struct()
    rc = lib().gc_compress_multi(ctx.handle, grad.data_ptr(), _grad_dtype(grad), residual.data_ptr(),
                                 off.ctypes.data, kk.ctypes.data, T, int(block), ctypes.byref(st),
                                 _stream_ptr(stream, grad.device))
    _check(rc, "gc_compress_multi")
    return out


def _buf_array(bufs: List[CompressedBuf]):
    arr = (_GcBuf * len(bufs))()
    for i, b in enumerate(bufs):
        arr[i] = b.struct()
    return arr


def decompress_sum(ctx: Context, bufs: List[CompressedBuf], n: int, out: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_sum: dense fp32 sum of W workers' compressed gradients (worker order, fp32)."""
    dev = bufs[0].q.device
    if out is None:
        out = torch.empty(int(n), dtype=torch.float32, device=dev)
    _check_dev(out, "out", torch.float32)
    arr = _buf_array(bufs)
    rc = lib().gc_decompress_sum(ctx.handle, arr, len(bufs), out.data_ptr(), int(n), _stream_ptr(stream, dev))
    _check(rc, "gc_decompress_sum")
    return out


def decompress_sum_static(ctx: Context, bufs: List[CompressedBuf], n: int, out: torch.Tensor,
                          stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_sum_static: the same aggregate without any allocation (static device scratch of
    GC_STATIC_SCRATCH_BYTES; larger calls raise GC_ERR_UNSUPPORTED). `out` must be given."""
    _check_dev(out, "out", torch.float32)
    arr = _buf_array(bufs)
    rc = lib().gc_decompress_sum_static(ctx.handle, arr, len(bufs), out.data_ptr(), int(n),
                                        _stream_ptr(stream, out.device))
    _check(rc, "gc_decompress_sum_static")
    return out


def decompress_sum_multi(ctx: Context, bufs: List[CompressedBuf], ks: Sequence[int], n: int,
                         out: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_sum_multi: the same for buffers written by compress_multi."""
    dev = bufs[0].q.device
    if out is None:
        out = torch.empty(int(n), dtype=torch.float32, device=dev)
    _check_dev(out, "out", torch.float32)
    kk = np.ascontiguousarray(ks, dtype=np.int64)
    arr = _buf_array(bufs)
    rc = lib().gc_decompress_sum_multi(ctx.handle, arr, len(bufs), kk.ctypes.data, kk.shape[0], out.data_ptr(),
                                       int(n), _stream_ptr(stream, dev))
    _check(rc, "gc_decompress_sum_multi")
    return out


def _kt(ks):
    if ks is None:
        return None, 0, None
    kk = np.ascontiguousarray(ks, dtype=np.int64)
    return kk.ctypes.data, kk.shape[0], kk


def decompress_sum_weighted(ctx: Context, bufs: List[CompressedBuf], staleness: Sequence[int], n: int,
                            out: Optional[torch.Tensor] = None, ks: Optional[Sequence[int]] = None,
                            stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_sum_weighted: worker w's contribution divided by 1 + staleness[w] (Eq. 12)."""
    dev = bufs[0].q.device
    if out is None:
        out = torch.empty(int(n), dtype=torch.float32, device=dev)
    _check_dev(out, "out", torch.float32)
    st = np.ascontiguousarray(staleness, dtype=np.int32)
    if st.shape[0] != len(bufs):
        raise ValueError("one staleness per buffer")
    kp, T, _keep = _kt(ks)
    rc = lib().gc_decompress_sum_weighted(ctx.handle, _buf_array(bufs), len(bufs), kp, T, st.ctypes.data,
                                          out.data_ptr(), int(n), _stream_ptr(stream, dev))
    _check(rc, "gc_decompress_sum_weighted")
    return out


def decompress_apply(ctx: Context, bufs: List[CompressedBuf], theta: torch.Tensor, step: float,
                     staleness: Optional[Sequence[int]] = None, ks: Optional[Sequence[int]] = None,
                     stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_apply: theta -= step * aggregate, touching only the positions the buffers name."""
    _check_dev(theta, "theta", torch.float32)
    st = None if staleness is None else np.ascontiguousarray(staleness, dtype=np.int32)
    if st is not None and st.shape[0] != len(bufs):
        raise ValueError("one staleness per buffer")
    kp, T, _keep = _kt(ks)
    rc = lib().gc_decompress_apply(ctx.handle, _buf_array(bufs), len(bufs), kp, T,
                                   None if st is None else st.ctypes.data, theta.data_ptr(), float(step),
                                   theta.numel(), _stream_ptr(stream, theta.device))
    _check(rc, "gc_decompress_apply")
    return theta


def compress_rows(ctx: Context, vals: torch.Tensor, residual_table: torch.Tensor, rows: torch.Tensor, k: int,
                  block: int, out: Optional[CompressedBuf] = None, index_bits: Optional[int] = None,
                  stream: Optional[torch.cuda.Stream] = None, codec: int = GC_CODEC_INT8) -> CompressedBuf:
    """gc_compress_rows: one step on the touched rows of a table-shaped residual (R x D, updated in place).
    vals: U*D values, rows: U ascending unique int64 row ids on the device. Indices come out as
    positions in the table."""
    _check_dev(vals, "vals")
    _check_dev(residual_table, "residual_table", torch.float32)
    _check_dev(rows, "rows", torch.int64)
    if residual_table.dim() != 2:
        raise ValueError("residual_table must be (R, D)")
    R, D = residual_table.shape
    U = rows.numel()
    if vals.numel() != U * D:
        raise ValueError("vals must hold U * D entries")
    if index_bits is None:
        index_bits = 64 if R * D > (1 << 32) else 32
    if out is None:
        kk = max(int(k), 0)
        out = CompressedBuf.allocate(R * D, kk, num_scales(kk, block), block, index_bits, vals.device, codec)
    st = out.struct()
    rc = lib().gc_compress_rows(ctx.handle, vals.data_ptr(), _grad_dtype(vals), residual_table.data_ptr(),
                                rows.data_ptr(), U, D, R, int(k), int(block), ctypes.byref(st),
                                _stream_ptr(stream, vals.device))
    _check(rc, "gc_compress_rows")
    return out


def decompress_sum_rows(ctx: Context, bufs: List[CompressedBuf], urows: torch.Tensor, D: int,
                        staleness: Optional[Sequence[int]] = None, out: Optional[torch.Tensor] = None,
                        stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_sum_rows: the aggregate of row-sparse buffers on the rows `urows` (ascending unique
    int64 on the device, containing every touched row). Returns (len(urows), D) fp32."""
    _check_dev(urows, "urows", torch.int64)
    Ru = urows.numel()
    if out is None:
        out = torch.empty((Ru, int(D)), dtype=torch.float32, device=urows.device)
    _check_dev(out, "out", torch.float32)
    st = None if staleness is None else np.ascontiguousarray(staleness, dtype=np.int32)
    if st is not None and st.shape[0] != len(bufs):
        raise ValueError("one staleness per buffer")
    rc = lib().gc_decompress_sum_rows(ctx.handle, _buf_array(bufs), len(bufs), urows.data_ptr(), Ru, int(D),
                                      None if st is None else st.ctypes.data, out.data_ptr(),
                                      _stream_ptr(stream, urows.device))
    _check(rc, "gc_decompress_sum_rows")
    return out


def compress_dense(ctx: Context, grad: torch.Tensor, residual: torch.Tensor, block: int,
                   codec: int = GC_CODEC_SIGN1, q: Optional[torch.Tensor] = None,
                   scales: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """gc_compress_dense: every entry coded (no indices); `residual` is updated in place.
    Returns (q, scales)."""
    _check_dev(grad, "grad")
    _check_dev(residual, "residual", torch.float32)
    n = grad.numel()
    if residual.numel() != n:
        raise ValueError("grad and residual differ in length")
    if q is None:
        nq = num_code_bytes(n, max(int(block), 1), codec)
        q = torch.empty(max(nq, 1), dtype=torch.int8, device=grad.device)[:nq]
    if scales is None:
        ns = num_scales(n, block)
        scales = torch.empty(max(ns, 1), dtype=torch.float32, device=grad.device)[:ns]
    _check_dev(q, "q", torch.int8)
    _check_dev(scales, "scales", torch.float32)
    rc = lib().gc_compress_dense(ctx.handle, grad.data_ptr(), _grad_dtype(grad), residual.data_ptr(), n, int(block),
                                 int(codec), q.data_ptr(), scales.data_ptr(), _stream_ptr(stream, grad.device))
    _check(rc, "gc_compress_dense")
    return q, scales


def _ptr_array(tensors: Sequence[torch.Tensor]):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def decompress_sum_dense(ctx: Context, qs: Sequence[torch.Tensor], scales: Sequence[torch.Tensor], n: int,
                         block: int, codec: int = GC_CODEC_SIGN1, staleness: Optional[Sequence[int]] = None,
                         out: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_sum_dense: fp32 sum, in worker order, of W workers' dense codes."""
    if len(qs) != len(scales):
        raise ValueError("one scales tensor per code tensor")
    dev = qs[0].device
    if out is None:
        out = torch.empty(int(n), dtype=torch.float32, device=dev)
    _check_dev(out, "out", torch.float32)
    st = None if staleness is None else np.ascontiguousarray(staleness, dtype=np.int32)
    if st is not None and st.shape[0] != len(qs):
        raise ValueError("one staleness per worker")
    rc = lib().gc_decompress_sum_dense(ctx.handle, _ptr_array(qs), _ptr_array(scales), len(qs), int(block),
                                       int(codec), None if st is None else st.ctypes.data, out.data_ptr(),
                                       int(n), _stream_ptr(stream, dev))
    _check(rc, "gc_decompress_sum_dense")
    return out


def decompress_apply_dense(ctx: Context, qs: Sequence[torch.Tensor], scales: Sequence[torch.Tensor],
                           theta: torch.Tensor, step: float, block: int, codec: int = GC_CODEC_SIGN1,
                           staleness: Optional[Sequence[int]] = None,
                           stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """gc_decompress_apply_dense: theta -= step * aggregate of the dense codes (Eq. 9)."""
    if len(qs) != len(scales):
        raise ValueError("one scales tensor per code tensor")
    _check_dev(theta, "theta", torch.float32)
    st = None if staleness is None else np.ascontiguousarray(staleness, dtype=np.int32)
    if st is not None and st.shape[0] != len(qs):
        raise ValueError("one staleness per worker")
    rc = lib().gc_decompress_apply_dense(ctx.handle, _ptr_array(qs), _ptr_array(scales), len(qs), int(block),
                                         int(codec), None if st is None else st.ctypes.data, theta.data_ptr(),
                                         float(step), theta.numel(), _stream_ptr(stream, theta.device))
    _check(rc, "gc_decompress_apply_dense")
    return theta


def sync_status(ctx: Context, stream: Optional[torch.cuda.Stream] = None, raise_on_error: bool = True) -> int:
    """gc_sync_status: wait for the stream; GC_ERR_NONFINITE if a compress call kept Inf/NaN."""
    s = stream if stream is not None else torch.cuda.current_stream(ctx.device)
    rc = lib().gc_sync_status(ctx.handle, int(s.cuda_stream))
    if raise_on_error:
        _check(rc, "gc_sync_status")
    return rc


def last_stats(ctx: Context) -> dict:
    st = _GcStats()
    _check(lib().gc_last_stats(ctx.handle, ctypes.byref(st)), "gc_last_stats")
    return {"tensors": st.tensors, "tensors_sampled": st.tensors_sampled,
            "tensors_fallback": st.tensors_fallback, "candidates": st.candidates}
