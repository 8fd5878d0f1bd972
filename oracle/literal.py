"""Literal pure-Python transcriptions of the oracle's definitions, for tiny inputs.

TEST INFRASTRUCTURE ONLY.  Everything here is written for obviousness, not speed: Python
sets, dicts and big integers, quadratic loops.  The compiled oracle (``oracle.cpp``) is
checked against these on small random inputs; these in turn are checked against
hand-worked examples and closed forms in the tests.
"""
from __future__ import annotations

import numpy as np


def f16_bits_to_float(h: int) -> float:
    """IEEE binary16 bit pattern -> Python float (exact)."""
    s, e, f = h >> 15, (h >> 10) & 31, h & 1023
    if e == 0:
        v = f * 2.0 ** -24
    elif e == 31:
        v = float("nan") if f else float("inf")
    else:
        v = (1024 + f) * 2.0 ** (e - 25)
    return -v if s else v


def spmm_dense(M, K, rowptr, colidx, vals, B):
    """Brute force: scatter A into a dense fp64 M x K array, then a dense matmul."""
    A = np.zeros((M, K), np.float64)
    for i in range(M):
        for p in range(rowptr[i], rowptr[i + 1]):
            A[i, colidx[p]] += f16_bits_to_float(int(vals[p]))
    Bd = np.array([[f16_bits_to_float(int(x)) for x in row] for row in B], np.float64).reshape(K, -1)
    return A @ Bd, np.abs(A) @ np.abs(Bd)


# ----------------------------------------------------------------------------- tile format
def encode(rowptr, colidx, vals, perm, WH, TW):
    """Bitmap tile format (paper Section 3.3) for WH x TW tiles; bitmaps are Python ints.

    Returns dict(row_window_offset, tc_offset, sparse_a_to_b, bitmaps, vals).
    """
    M = len(rowptr) - 1
    perm = list(range(M)) if perm is None else list(perm)
    rwo, tco, a2b, bitmaps, packed = [0], [0], [], [], []
    for w0 in range(0, M, WH):
        rows = [perm[r] for r in range(w0, min(M, w0 + WH))]
        cols = sorted({int(colidx[p]) for i in rows for p in range(rowptr[i], rowptr[i + 1])})
        ntile = -(-len(cols) // TW)
        for t in range(ntile):
            tcols = cols[t * TW:(t + 1) * TW]
            a2b += tcols + [cols[-1]] * (TW - len(tcols))
            entries = {}  # bit index -> value
            for rl, i in enumerate(rows):
                for p in range(rowptr[i], rowptr[i + 1]):
                    if int(colidx[p]) in tcols:
                        bit = rl * TW + tcols.index(int(colidx[p]))
                        assert bit not in entries, "duplicate column in a row"
                        entries[bit] = int(vals[p])
            bitmaps.append(sum(1 << b for b in entries))
            packed += [entries[b] for b in sorted(entries)]
            tco.append(len(packed))
        rwo.append(len(bitmaps))
    return dict(row_window_offset=rwo, tc_offset=tco, sparse_a_to_b=a2b, bitmaps=bitmaps, vals=packed)


def bitmap_words(bitmaps, WH, TW):
    """Python-int bitmaps -> flat list of 64-bit words (word k holds bits [64k, 64k+64))."""
    nw = -(-(WH * TW) // 64)
    return [(b >> (64 * k)) & (2 ** 64 - 1) for b in bitmaps for k in range(nw)]


def decode(fmt, M, WH, TW):
    """Position p of tile g holds vals[tc_offset[g] + popcount(bitmap & ((1<<p)-1))] if bit p is set."""
    rows = []
    for r in range(M):
        w, rl = divmod(r, WH)
        row = []
        for g in range(fmt["row_window_offset"][w], fmt["row_window_offset"][w + 1]):
            bm = fmt["bitmaps"][g]
            for c in range(TW):
                p = rl * TW + c
                if bm >> p & 1:
                    off = fmt["tc_offset"][g] + bin(bm & ((1 << p) - 1)).count("1")
                    row.append((fmt["sparse_a_to_b"][g * TW + c], fmt["vals"][off]))
        rows.append(row)
    return rows


# ------------------------------------------------------------------------------ reordering
def graph(rowptr, colidx):
    """Undirected unit-weight graph of the pattern of A + A^T without the diagonal."""
    M = len(rowptr) - 1
    adj = [set() for _ in range(M)]
    for i in range(M):
        for p in range(rowptr[i], rowptr[i + 1]):
            j = int(colidx[p])
            if j != i:
                adj[i].add(j)
                adj[j].add(i)
    return adj


def dendrogram(rowptr, colidx):
    """Algorithm 1 Step I, recomputing every community quantity from scratch at each turn."""
    adj = graph(rowptr, colidx)
    M = len(adj)
    deg = [len(a) for a in adj]
    two_m = sum(deg)
    label = list(range(M))          # community (root id) of each vertex
    parent = [-1] * M
    child_order = [0] * M
    nchild = [0] * M
    for v in sorted(range(M), key=lambda x: (deg[x], x)):
        members = [x for x in range(M) if label[x] == v]
        d_v = sum(deg[x] for x in members)
        w = {}
        for x in members:
            for y in adj[x]:
                if label[y] != v:
                    w[label[y]] = w.get(label[y], 0) + 1
        best, best_s = -1, 0
        for u in sorted(w):
            d_u = sum(deg[x] for x in range(M) if label[x] == u)
            s = w[u] * two_m - d_u * d_v
            if best < 0 or s > best_s:
                best, best_s = u, s
        if best >= 0 and best_s > 0:
            parent[v] = best
            child_order[v] = nchild[best]
            nchild[best] += 1
            for x in members:
                label[x] = best
    return parent, child_order


def leaf_sequence(parent, child_order):
    M = len(parent)
    children = [[] for _ in range(M)]
    for v in range(M):
        if parent[v] >= 0:
            children[parent[v]].append((child_order[v], v))
    trees = []

    def emit(r, out):
        out.append(r)
        for _, c in sorted(children[r]):
            emit(c, out)

    import sys
    sys.setrecursionlimit(max(10000, 4 * M + 100))
    for r in range(M):
        if parent[r] < 0:
            out = []
            emit(r, out)
            trees.append(out)
    return trees


def ordering(rowptr, colidx, parent, child_order, seg_len):
    """Algorithm 1 Step II with the segment-limited candidate search."""
    M = len(parent)
    cols = [set(int(c) for c in colidx[rowptr[i]:rowptr[i + 1]]) for i in range(M)]
    perm = []
    for tree in leaf_sequence(parent, child_order):
        for s0 in range(0, len(tree), seg_len):
            seg = tree[s0:s0 + seg_len]
            visited = set()
            for first in seg:
                if first in visited:
                    continue
                v = first
                while True:
                    visited.add(v)
                    perm.append(v)
                    best, best_n = None, 0
                    for u in seg:                       # sequence order: earliest wins ties
                        if u not in visited:
                            n = len(cols[u] & cols[v])
                            if n > best_n:
                                best, best_n = u, n
                    if best is None:
                        break
                    v = best
    iperm = [0] * M
    for new, old in enumerate(perm):
        iperm[old] = new
    return perm, iperm


def ibd(row_window_offset):
    """Eq. 3: mean absolute deviation of tiles per window."""
    t = np.diff(np.asarray(row_window_offset, np.float64))
    return float(np.abs(t - t.mean()).mean()) if len(t) else 0.0
