"""Small helpers for the tests (no method arithmetic)."""
import json
import os

import numpy as np


def csr_from_rows(rows, vals=None):
    """rows: list of column lists.  vals: list of numbers per entry (default: p+1), stored as fp16 bits."""
    rowptr = np.zeros(len(rows) + 1, np.int32)
    for i, r in enumerate(rows):
        rowptr[i + 1] = rowptr[i] + len(r)
    colidx = np.array([c for r in rows for c in r], np.int32)
    nnz = len(colidx)
    v = np.arange(1, nnz + 1, dtype=np.float16) if vals is None else np.asarray(vals, np.float16)
    return rowptr, colidx, v.view(np.uint16).copy()


def csr_from_edges(M, edges):
    rows = [set() for _ in range(M)]
    for a, b in edges:
        rows[a].add(b)
        rows[b].add(a)
    return csr_from_rows([sorted(r) for r in rows])


def random_csr(rng, M, K, density, empty_row_frac=0.1):
    rows = []
    for _ in range(M):
        if rng.random() < empty_row_frac:
            rows.append([])
        else:
            n = rng.binomial(K, density)
            rows.append(sorted(rng.choice(K, size=min(n, K), replace=False).tolist()))
    nnz = sum(len(r) for r in rows)
    vals = rng.uniform(-1, 1, nnz).astype(np.float16)
    return csr_from_rows(rows, vals)


def random_sym_csr(rng, M, avg_deg):
    edges = set()
    for _ in range(int(M * avg_deg / 2)):
        a, b = rng.integers(0, M, 2)
        if a != b:
            edges.add((int(min(a, b)), int(max(a, b))))
    return csr_from_edges(M, edges)


def load_golden(name):
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)) as f:
        return json.load(f)


def f16(a):
    return np.asarray(a, np.float16).view(np.uint16).copy()


def bf16(a):
    """float -> bfloat16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_to_f64(bits):
    with np.errstate(invalid="ignore"):                      # signalling NaN patterns are fine here
        return (np.asarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
