"""ctypes loader for the CPU oracle (oracle/gc_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg. The product package never imports this module.
It does argument marshalling for numpy arrays and nothing else.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gc_oracle.cpp")
_LIB = os.path.join(_HERE, "libgc_oracle.so")

OK, ERR_INVALID_ARG, ERR_NONFINITE = 0, 1, 4
F32, BF16 = 0, 1
INT8, SIGN1 = 0, 1  # value codes


def build(force: bool = False) -> str:
    """Compile the oracle with contraction off so every fp32 op rounds on its own."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared",
               "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.gco_k_from_density.restype = ctypes.c_int64
        L.gco_k_from_density.argtypes = [ctypes.c_int64, ctypes.c_double]
        L.gco_compress.restype = ctypes.c_int
        L.gco_compress.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int64,
                                   ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p,
                                   ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        L.gco_compress_multi.restype = ctypes.c_int
        L.gco_compress_multi.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                         ctypes.c_void_p, ctypes.c_void_p]
        L.gco_decompress_sum.restype = ctypes.c_int
        L.gco_decompress_sum.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                         ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                         ctypes.c_void_p, ctypes.c_int64]
        L.gco_decompress_sum_weighted.restype = ctypes.c_int
        L.gco_decompress_sum_weighted.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                                  ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        L.gco_num_code_bytes.restype = ctypes.c_int64
        L.gco_num_code_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        L.gco_compress_codec.restype = ctypes.c_int
        L.gco_compress_codec.argtypes = L.gco_compress.argtypes + [ctypes.c_int32]
        L.gco_compress_multi_codec.restype = ctypes.c_int
        L.gco_compress_multi_codec.argtypes = L.gco_compress_multi.argtypes + [ctypes.c_int32]
        L.gco_decompress_sum_codec.restype = ctypes.c_int
        L.gco_decompress_sum_codec.argtypes = L.gco_decompress_sum_weighted.argtypes + [ctypes.c_int32]
        L.gco_compress_rows.restype = ctypes.c_int
        L.gco_compress_rows.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.c_int32]
        L.gco_decompress_sum_rows.restype = ctypes.c_int
        L.gco_decompress_sum_rows.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                              ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_int32]
        L.gco_apply.restype = ctypes.c_int
        L.gco_apply.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_int64]
        _lib = L
    return _lib


def k_from_density(n: int, density: float) -> int:
    return int(lib().gco_k_from_density(int(n), float(density)))


def _grad_dtype(g: np.ndarray) -> int:
    if g.dtype == np.float32:
        return F32
    if g.dtype == np.uint16:  # bf16 bit patterns
        return BF16
    raise TypeError("gradient must be float32 or uint16 (bf16 bit patterns)")


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def num_code_bytes(k: int, block: int, codec: int = INT8) -> int:
    return int(lib().gco_num_code_bytes(int(k), int(block), int(codec)))


def compress(g: np.ndarray, e: np.ndarray, k: int, block: int, index_bits: int = 32, codec: int = INT8):
    """One error-feedback step. `e` (float32) is updated IN PLACE to r_{t+1}.

    Returns (status, idx, q, scales); with codec=SIGN1 `q` holds the packed sign bytes."""
    n = g.shape[0]
    assert e.dtype == np.float32 and e.shape[0] == n
    kk = max(int(k), 0)
    idx = np.zeros(kk, dtype=np.uint32 if index_bits == 32 else np.uint64)
    q = np.zeros(max(num_code_bytes(kk, max(block, 1), codec), 0), dtype=np.int8)
    nb = (kk + block - 1) // block if block > 0 else 0
    s = np.zeros(max(nb, 1), dtype=np.float32)
    # zero-length arrays still need a non-null pointer for the argument check
    pad = np.zeros(1, dtype=np.uint64)
    rc = lib().gco_compress_codec(_ptr(g), _grad_dtype(g), _ptr(e), n, int(k), int(block),
                                  _ptr(idx) if kk else _ptr(pad), index_bits,
                                  _ptr(q) if q.size else _ptr(pad), _ptr(s), int(codec))
    return rc, idx, q, s[:nb]


def compress_rows(vals: np.ndarray, e_table: np.ndarray, rows: np.ndarray, k: int, block: int,
                  index_bits: int = 64, codec: int = INT8):
    """One step on the touched rows of a table-shaped residual. vals: (U*D,) values of the touched
    rows, e_table: (R, D) float32 updated IN PLACE on those rows, rows: (U,) ascending unique int64.
    Returns (status, idx, q, scales); idx are positions in the table (row * D + column)."""
    assert e_table.dtype == np.float32 and e_table.ndim == 2 and e_table.flags["C_CONTIGUOUS"]
    R, D = e_table.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    U = rows.shape[0]
    assert vals.shape[0] == U * D
    kk = max(int(k), 0)
    idx = np.zeros(max(kk, 1), dtype=np.uint32 if index_bits == 32 else np.uint64)
    q = np.zeros(max(num_code_bytes(kk, max(block, 1), codec), 1), dtype=np.int8)
    nb = (kk + block - 1) // block if block > 0 else 0
    s = np.zeros(max(nb, 1), dtype=np.float32)
    rc = lib().gco_compress_rows(_ptr(vals), _grad_dtype(vals), _ptr(e_table), _ptr(rows), U, D, R, int(k),
                                 int(block), _ptr(idx), index_bits, _ptr(q), _ptr(s), int(codec))
    return rc, idx[:kk], q[:max(num_code_bytes(kk, max(block, 1), codec), 0)], s[:nb]


def compress_multi(g: np.ndarray, e: np.ndarray, offsets, ks, block: int, index_bits: int = 32,
                   codec: int = INT8):
    """Per-tensor top-k over a flat concatenation. Returns (status, idx, q, scales)."""
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    ks = np.ascontiguousarray(ks, dtype=np.int64)
    T = ks.shape[0]
    ktot = int(ks.sum())
    stot = int(((ks + block - 1) // block).sum())
    idx = np.zeros(ktot, dtype=np.uint32 if index_bits == 32 else np.uint64)
    q = np.zeros(sum(num_code_bytes(int(x), block, codec) for x in ks), dtype=np.int8)
    s = np.zeros(stot, dtype=np.float32)
    rc = lib().gco_compress_multi_codec(_ptr(g), _grad_dtype(g), _ptr(e), _ptr(offsets), _ptr(ks), T,
                                        int(block), _ptr(idx), index_bits, _ptr(q), _ptr(s), int(codec))
    return rc, idx, q, s


def decompress_sum(bufs, n: int, block: int, ktensor=None, staleness=None, codec: int = INT8):
    """bufs: list of (idx, q, scales) numpy triples, one per worker. Returns (status, out).
    staleness: optional per-worker integers (Eq. 12 damping)."""
    W = len(bufs)
    index_bits = 32 if bufs[0][0].dtype == np.uint32 else 64
    PA = ctypes.c_void_p * W
    ia = PA(*[_ptr(b[0]) for b in bufs])
    qa = PA(*[_ptr(b[1]) for b in bufs])
    sa = PA(*[_ptr(b[2]) for b in bufs])
    kc = np.array([b[0].shape[0] for b in bufs], dtype=np.int64)
    out = np.empty(n, dtype=np.float32)
    if ktensor is not None:
        kt = np.ascontiguousarray(ktensor, dtype=np.int64)
        ktp, T = _ptr(kt), kt.shape[0]
    else:
        ktp, T = None, 0
    if staleness is not None:
        st = np.ascontiguousarray(staleness, dtype=np.int32)
        assert st.shape[0] == W
        stp = _ptr(st)
    else:
        stp = None
    rc = lib().gco_decompress_sum_codec(W, ctypes.addressof(ia), ctypes.addressof(qa),
                                        ctypes.addressof(sa), _ptr(kc), int(block), index_bits, ktp, T,
                                        stp, _ptr(out), int(n), int(codec))
    return rc, out


def decompress_sum_rows(bufs, urows, D: int, block: int, staleness=None, codec: int = INT8):
    """bufs: (idx, q, scales) triples whose idx are table positions (row * D + column); urows:
    ascending unique rows containing every touched row. Returns (status, out) with out (len(urows), D)."""
    W = len(bufs)
    index_bits = 32 if bufs[0][0].dtype == np.uint32 else 64
    PA = ctypes.c_void_p * W
    ia = PA(*[_ptr(b[0]) for b in bufs])
    qa = PA(*[_ptr(b[1]) for b in bufs])
    sa = PA(*[_ptr(b[2]) for b in bufs])
    kc = np.array([b[0].shape[0] for b in bufs], dtype=np.int64)
    ur = np.ascontiguousarray(urows, dtype=np.int64)
    out = np.empty((ur.shape[0], int(D)), dtype=np.float32)
    if staleness is not None:
        st = np.ascontiguousarray(staleness, dtype=np.int32)
        assert st.shape[0] == W
        stp = _ptr(st)
    else:
        stp = None
    rc = lib().gco_decompress_sum_rows(W, ctypes.addressof(ia), ctypes.addressof(qa), ctypes.addressof(sa),
                                       _ptr(kc), int(block), index_bits, _ptr(ur), ur.shape[0], int(D), stp,
                                       _ptr(out), int(codec))
    return rc, out


def apply(theta: np.ndarray, S: np.ndarray, step: float) -> int:
    """theta <- theta - step * S in place (Eq. 9 with eta / P = step)."""
    assert theta.dtype == np.float32 and S.dtype == np.float32 and theta.shape == S.shape
    return lib().gco_apply(_ptr(theta), _ptr(S), float(step), theta.shape[0])
