"""CPU oracle for the Acc-SpMM hot path.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``oracle.cpp`` (fp64 SpMM, tile-format encode/decode, the two
steps of the reordering, the imbalance degree) plus ``literal.py``, a pure-Python
transcription of the same definitions for tiny inputs.  Only tests, the smoke check and
the benchmark's ``cpu_baseline`` leg import this package; the GPU library never does and
shares no code with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

SEG_LEN = 1024  # default segment length of the ordering step


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["g++", "-O2", "-fopenmp", "-std=c++17", "-shared", "-fPIC", _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        L.orc_f16_to_f64.restype = ctypes.c_double
        L.orc_f16_to_f64.argtypes = [ctypes.c_uint16]
        L.orc_bf16_to_f64.restype = ctypes.c_double
        L.orc_bf16_to_f64.argtypes = [ctypes.c_uint16]
        L.orc_spmm_rows.restype = None
        L.orc_spmm_rows.argtypes = [i64, vp, i64, vp, vp, vp, vp, vp, vp]
        L.orc_sddmm.restype = None
        L.orc_sddmm.argtypes = [i64, i64, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int]
        L.orc_spmm_rows_typed.restype = None
        L.orc_spmm_rows_typed.argtypes = [i64, vp, i64, vp, vp, vp, vp, vp, vp, ctypes.c_int]
        L.orc_encode.restype = i64
        L.orc_encode.argtypes = [i64, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp]
        L.orc_decode.restype = None
        L.orc_decode.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.orc_dendrogram.restype = None
        L.orc_dendrogram.argtypes = [i64, vp, vp, vp, vp]
        L.orc_ordering.restype = None
        L.orc_ordering.argtypes = [i64, vp, vp, vp, vp, i32, vp, vp, vp, vp]
        L.orc_set_progress.restype = None
        L.orc_set_progress.argtypes = [i64]
        L.orc_ibd.restype = ctypes.c_double
        L.orc_ibd.argtypes = [i64, vp]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _u16(a):
    return np.ascontiguousarray(a, dtype=np.uint16)


def spmm(rowptr, colidx, vals, B, rows=None, want_bound=True, value_type="f16"):
    """fp64 C = A.B and bound = |A|.|B| for all rows, or for the given row indices.
    `vals` and `B` are 16-bit patterns of `value_type` ("f16" = IEEE binary16, "bf16")."""
    rowptr, colidx, vals, B = _i32(rowptr), _i32(colidx), _u16(vals), _u16(B)
    N = B.shape[1]
    if rows is None:
        n, rp = len(rowptr) - 1, None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n, rp = len(rows), rows.ctypes.data
    C = np.empty((n, N), np.float64)
    bound = np.empty((n, N), np.float64) if want_bound else None
    _load().orc_spmm_rows_typed(n, rp, N, _p(rowptr), _p(colidx), _p(vals), _p(B), _p(C), _p(bound),
                                {"f16": 0, "bf16": 1}[value_type])
    return C, bound


def sddmm(rowptr, colidx, X, Y, vals=None, value_type="f16"):
    """fp64 out[p] = (vals[p] if given) * <X[i_p], Y[j_p]> for every stored entry p, and
    bound[p] = |vals[p]| * <|X[i_p]|, |Y[j_p]|>.  X: M x N, Y: K x N bit patterns."""
    rowptr, colidx, X, Y = _i32(rowptr), _i32(colidx), _u16(X), _u16(Y)
    vals = None if vals is None else _u16(vals)
    M, N = len(rowptr) - 1, X.shape[1]
    assert X.shape[0] == M and Y.shape[1] == N
    out = np.empty(len(colidx), np.float64)
    bound = np.empty(len(colidx), np.float64)
    _load().orc_sddmm(M, N, _p(rowptr), _p(colidx), _p(vals), _p(X), _p(Y), _p(out), _p(bound),
                      {"f16": 0, "bf16": 1}[value_type])
    return out, bound


def encode(rowptr, colidx, vals, perm=None, WH=16, TW=16):
    """Tile format of the (row-reordered) matrix.  Returns a dict of the five arrays."""
    rowptr, colidx, vals = _i32(rowptr), _i32(colidx), _u16(vals)
    perm = None if perm is None else _i32(perm)
    M = len(rowptr) - 1
    L = _load()
    T = L.orc_encode(M, _p(rowptr), _p(colidx), _p(vals), _p(perm), WH, TW, None, None, None, None, None)
    W = (M + WH - 1) // WH
    NW = (WH * TW + 63) // 64
    out = dict(
        WH=WH, TW=TW, M=M,
        row_window_offset=np.zeros(W + 1, np.int32),
        tc_offset=np.zeros(T + 1, np.int32),
        sparse_a_to_b=np.zeros(T * TW, np.int32),
        tc_local_bit=np.zeros(T * NW, np.uint64),
        vals=np.zeros(len(vals), np.uint16),
    )
    r = L.orc_encode(M, _p(rowptr), _p(colidx), _p(vals), _p(perm), WH, TW, _p(out["row_window_offset"]),
                     _p(out["tc_offset"]), _p(out["sparse_a_to_b"]), _p(out["tc_local_bit"]), _p(out["vals"]))
    if r < 0:
        raise ValueError("duplicate column inside a row")
    return out


def decode(fmt):
    """Inverse of encode: CSR (rowptr, colidx, vals) of the reordered matrix."""
    M = fmt["M"]
    nnz = int(fmt["tc_offset"][-1]) if len(fmt["tc_offset"]) else 0
    rowptr = np.zeros(M + 1, np.int32)
    colidx = np.zeros(nnz, np.int32)
    vals = np.zeros(nnz, np.uint16)
    _load().orc_decode(M, fmt["WH"], fmt["TW"], _p(fmt["row_window_offset"]), _p(fmt["tc_offset"]),
                       _p(fmt["sparse_a_to_b"]), _p(fmt["tc_local_bit"]), _p(fmt["vals"]),
                       _p(rowptr), _p(colidx), _p(vals))
    return rowptr, colidx, vals


def set_progress(every):
    """Step I prints a line on stderr every `every` vertices (0: silent).  For runs that take minutes."""
    _load().orc_set_progress(int(every))


def dendrogram(rowptr, colidx):
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    M = len(rowptr) - 1
    parent = np.empty(M, np.int32)
    child_order = np.empty(M, np.int32)
    _load().orc_dendrogram(M, _p(rowptr), _p(colidx), _p(parent), _p(child_order))
    return parent, child_order


def ordering(rowptr, colidx, parent, child_order, seg_len=SEG_LEN, details=False):
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    parent, child_order = _i32(parent), _i32(child_order)
    M = len(rowptr) - 1
    perm = np.empty(M, np.int32)
    iperm = np.empty(M, np.int32)
    seq = np.empty(M, np.int32)
    seg = np.full(M + 1, -1, np.int32)
    _load().orc_ordering(M, _p(rowptr), _p(colidx), _p(parent), _p(child_order), seg_len,
                         _p(perm), _p(iperm), _p(seq), _p(seg))
    if details:
        nseg = int(np.argmax(seg == M)) if M else 0
        return perm, iperm, seq, seg[: nseg + 1]
    return perm, iperm


def reorder(rowptr, colidx, seg_len=SEG_LEN):
    """perm (new -> old) and iperm (old -> new) of the data-affinity reordering."""
    parent, child_order = dendrogram(rowptr, colidx)
    return ordering(rowptr, colidx, parent, child_order, seg_len)


def ibd(row_window_offset) -> float:
    rwo = _i32(row_window_offset)
    return float(_load().orc_ibd(len(rwo) - 1, _p(rwo)))


def within_bound(C_gpu, C_ref, bound, rel=2e-3, abs_=1e-5):
    """Elementwise acceptance test |C - C_ref| <= rel*bound + abs_.  Returns (ok, worst ratio)."""
    err = np.abs(C_gpu.astype(np.float64) - C_ref)
    lim = rel * bound + abs_
    ratio = float((err / lim).max()) if err.size else 0.0
    return bool(np.all(err <= lim)) and bool(np.isfinite(C_gpu).all()), ratio


def column_order(colidx, K):
    """Column order used for the rows of B: columns grouped by floor(log2(number of stored
    entries in the column)), groups by descending class, ascending column id inside a group,
    columns without entries last.  Returns (order, rank): order[j] = input column at plan
    position j, rank = its inverse.

    The paper only names column reordering with the matching row reordering of B as the step
    after row reordering (Section 4.3.1, conclusion) and gives no rule: this rule is the
    library's own, so it is PARITY UNPINNED against the paper; the tests pin it to this
    definition by brute force.  C = A.B does not depend on it."""
    colidx = np.asarray(colidx, np.int64)
    count = np.bincount(colidx, minlength=K)
    cls = np.full(K, -1, np.int64)
    used = count > 0
    cls[used] = np.floor(np.log2(count[used])).astype(np.int64)
    # exact for counts < 2^31: log2 of a power of two is exact in fp64, and other counts are
    # at least one part in 2^31 away from the next power of two
    order = np.argsort(-cls, kind="stable").astype(np.int32)
    rank = np.empty(K, np.int32)
    rank[order] = np.arange(K, dtype=np.int32)
    return order, rank
