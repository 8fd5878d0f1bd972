"""Seeded synthetic inputs shared by the oracle's tests and the GPU library's tests.

Nothing in here is part of the SpMM method: this module only draws random sparse
structure and random fp16 values (see ``gen.cpp``).  The five workloads stand in for
the graph and SuiteSparse matrices the Acc-SpMM paper evaluates on (Table 1; Section
4.1 uses feature widths 128..512), which are not redistributed here.

fp16 data is carried as ``numpy.uint16`` bit patterns (``.view(numpy.float16)`` to read).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.cpp")
_LIB = os.path.join(_HERE, "libworkloads.so")
_lib = None

SEED_BASE = 0xACC5B000


def build(force: bool = False) -> str:
    """Compile the generator library (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["g++", "-O3", "-fopenmp", "-std=c++17", "-shared", "-fPIC", _SRC, "-o", _LIB]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i64, i32, u64, f32, f64 = (
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_float, ctypes.c_double)
        L.wl_csr_nnz.restype = i64
        L.wl_csr_nnz.argtypes = [vp]
        L.wl_csr_rows.restype = i64
        L.wl_csr_rows.argtypes = [vp]
        L.wl_csr_copy.restype = None
        L.wl_csr_copy.argtypes = [vp, vp, vp, vp]
        L.wl_csr_free.restype = None
        L.wl_csr_free.argtypes = [vp]
        L.wl_uniform.restype = vp
        L.wl_uniform.argtypes = [i64, i64, i32, u64, f32, f32]
        L.wl_rmat.restype = vp
        L.wl_rmat.argtypes = [i32, i64, f64, f64, f64, u64, i32, f32, f32]
        L.wl_stencil27.restype = vp
        L.wl_stencil27.argtypes = [i32, u64, f32, f32, f32]
        L.wl_sbm.restype = vp
        L.wl_sbm.argtypes = [i64, i32, f64, f64, u64, i32, f32, f32]
        L.wl_dense.restype = None
        L.wl_dense.argtypes = [i64, i64, u64, i32, f32, f32, vp]
        L.wl_f32_to_f16.restype = ctypes.c_uint16
        L.wl_f32_to_f16.argtypes = [f32]
        L.wl_rnd.restype = u64
        L.wl_rnd.argtypes = [u64, u64, u64]
        _lib = L
    return _lib


@dataclass
class Workload:
    """One SpMM problem: A (CSR, fp16 bits) and B (dense row-major fp16 bits)."""
    name: str
    M: int
    K: int
    N: int
    rowptr: np.ndarray   # int32[M+1]
    colidx: np.ndarray   # int32[nnz], ascending and distinct within each row
    vals: np.ndarray     # uint16[nnz]
    B: np.ndarray        # uint16[K, N]

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def _take(handle) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    L = _load()
    if not handle:
        raise ValueError("generator rejected its arguments")
    try:
        M, nnz = L.wl_csr_rows(handle), L.wl_csr_nnz(handle)
        rowptr = np.empty(M + 1, np.int32)
        colidx = np.empty(nnz, np.int32)
        vals = np.empty(nnz, np.uint16)
        L.wl_csr_copy(handle, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data)
    finally:
        L.wl_csr_free(handle)
    return rowptr, colidx, vals


def dense(rows: int, cols: int, seed: int, kind: str = "uniform", p0: float = -1.0, p1: float = 1.0) -> np.ndarray:
    """Dense fp16 matrix: kind 'uniform' draws U[p0,p1], 'normal' draws N(p0, p1^2)."""
    out = np.empty((rows, cols), np.uint16)
    if out.size:
        _load().wl_dense(rows, cols, seed, 0 if kind == "uniform" else 1, p0, p1, out.ctypes.data)
    return out


def uniform(M: int, K: int, per_row: int, seed: int, lo=-1.0, hi=1.0):
    return _take(_load().wl_uniform(M, K, per_row, seed, lo, hi))


def rmat(scale: int, n_samples: int, seed: int, symmetrize: bool, lo=0.0, hi=1.0, a=0.57, b=0.19, c=0.19):
    return _take(_load().wl_rmat(scale, n_samples, a, b, c, seed, int(symmetrize), lo, hi))


def stencil27(n: int, seed: int, diag=26.0, lo=-1.0, hi=1.0):
    return _take(_load().wl_stencil27(n, seed, diag, lo, hi))


def sbm(V: int, csize: int, p_in: float, inter_deg: float, seed: int, relabel: bool = True, lo=-1.0, hi=1.0):
    return _take(_load().wl_sbm(V, csize, p_in, inter_deg, seed, int(relabel), lo, hi))


CONFIG_NAMES = {
    1: "uniform-4096x8-N32",
    2: "rmat-2^20-deg16-sym-N128",
    3: "stencil27-128^3-N64",
    4: "sbm-2^18-c64-N256",
    5: "rmat-2^23-deg32-N128",
}


def config(cfg: int, shrink: int = 0, with_B: bool = True) -> Workload:
    """Workload `cfg` (1..5) of the benchmark set.

    `shrink` = s divides the number of rows by 2^s (2^(3*ceil(s/3)) for the stencil grid's
    volume, since the grid edge is halved) while keeping the recipe, the row-length
    distribution and N; shrink=0 is the full-size workload.
    """
    seed = SEED_BASE + cfg
    if cfg == 1:
        M = max(4096 >> shrink, 16)
        A = uniform(M, M, 8, seed)
        N, kind, p0, p1 = 32, "uniform", -1.0, 1.0
    elif cfg == 2:
        sc = max(20 - shrink, 4)
        A = rmat(sc, 8 << sc, seed, True)
        N, kind, p0, p1 = 128, "normal", 0.0, 1.0
    elif cfg == 3:
        n = max(128 >> ((shrink + 2) // 3), 2)
        A = stencil27(n, seed)
        N, kind, p0, p1 = 64, "uniform", -1.0, 1.0
    elif cfg == 4:
        V = max((1 << 18) >> shrink, 128)
        A = sbm(V, 64, 0.25, 4.0, seed, True)
        N, kind, p0, p1 = 256, "normal", 0.0, 1.0
    elif cfg == 5:
        sc = max(23 - shrink, 4)
        A = rmat(sc, 32 << sc, seed, False)
        N, kind, p0, p1 = 128, "normal", 0.0, 1.0
    else:
        raise ValueError("cfg must be 1..5")
    rowptr, colidx, vals = A
    M = len(rowptr) - 1
    B = dense(M, N, seed ^ 0xB, kind, p0, p1) if with_B else np.empty((0, N), np.uint16)
    name = CONFIG_NAMES[cfg] + (f"/shrink{shrink}" if shrink else "")
    return Workload(name, M, M, N, rowptr, colidx, vals, B)
