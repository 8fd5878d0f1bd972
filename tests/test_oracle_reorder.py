"""Pins for the reordering oracle (paper Section 3.2, Algorithm 1).

Parity with the paper's own worked example is unpinned (it lives in a figure that is not
available); the pins are hand-worked graphs, structural properties and a literal
pure-Python transcription.
"""
import numpy as np
import pytest

import oracle
from oracle import literal
from _util import csr_from_rows, csr_from_edges, random_sym_csr, random_csr, load_golden


def test_hand_worked_two_triangles():
    g = load_golden("reorder_two_triangles.json")
    rowptr, colidx, _ = csr_from_edges(g["M"], g["edges"])
    for dend in (oracle.dendrogram, literal.dendrogram):
        parent, child_order = dend(rowptr, colidx)
        assert list(parent) == g["parent"] and list(child_order) == g["child_order"]
    perm, iperm, seq, seg = oracle.ordering(rowptr, colidx, g["parent"], g["child_order"], 1024, details=True)
    assert list(seq) == g["leaf_sequence"] and list(seg) == [0, 3, 6]
    assert list(perm) == g["perm"]
    lperm, liperm = literal.ordering(rowptr, colidx, g["parent"], g["child_order"], 1024)
    assert lperm == g["perm"] and list(iperm) == liperm


def test_hand_worked_chain_with_ties_breaks_and_segments():
    g = load_golden("ordering_chain.json")
    rowptr, colidx, _ = csr_from_rows(g["rows"])
    for seg_len, key in ((6, "perm_seg6"), (3, "perm_seg3")):
        perm, iperm = oracle.ordering(rowptr, colidx, g["parent"], g["child_order"], seg_len)
        assert list(perm) == g[key]
        lperm, _ = literal.ordering(rowptr, colidx, g["parent"], g["child_order"], seg_len)
        assert lperm == g[key]
        assert [int(iperm[o]) for o in perm] == list(range(g["M"]))


def _special_graphs():
    star = [(0, i) for i in range(1, 12)]
    path = [(i, i + 1) for i in range(14)]
    clique = [(i, j) for i in range(7) for j in range(i + 1, 7)]
    two_cliques = clique + [(i + 7, j + 7) for i, j in clique] + [(0, 7)]
    return {"star": (12, star), "path": (15, path), "clique": (7, clique), "two_cliques": (14, two_cliques),
            "isolated": (5, []), "pair_plus_isolated": (6, [(4, 5)])}


@pytest.mark.parametrize("name", list(_special_graphs()))
def test_special_graphs_compiled_equals_literal(name):
    M, edges = _special_graphs()[name]
    rowptr, colidx, _ = csr_from_edges(M, edges)
    parent, child_order = oracle.dendrogram(rowptr, colidx)
    lparent, lchild = literal.dendrogram(rowptr, colidx)
    assert list(parent) == lparent and list(child_order) == lchild
    for seg_len in (3, 1024):
        perm, _ = oracle.ordering(rowptr, colidx, parent, child_order, seg_len)
        lperm, _ = literal.ordering(rowptr, colidx, lparent, lchild, seg_len)
        assert list(perm) == lperm
        assert sorted(perm) == list(range(M))


def test_clique_collapses_to_one_community_and_isolated_stay_roots():
    M, edges = _special_graphs()["two_cliques"]
    rowptr, colidx, _ = csr_from_edges(M, edges)
    parent, _ = oracle.dendrogram(rowptr, colidx)
    root = lambda x: x if parent[x] < 0 else root(parent[x])
    assert len({root(i) for i in range(7)}) == 1 and len({root(i) for i in range(7, 14)}) == 1
    assert root(0) != root(7)
    rowptr, colidx, _ = csr_from_edges(5, [])
    parent, _ = oracle.dendrogram(rowptr, colidx)
    assert list(parent) == [-1] * 5
    perm, _ = oracle.reorder(rowptr, colidx)
    assert list(perm) == [0, 1, 2, 3, 4]


@pytest.mark.parametrize("seed", range(8))
def test_random_graphs_compiled_equals_literal(seed):
    rng = np.random.default_rng(seed)
    M = int(rng.integers(20, 160))
    if seed % 2:
        rowptr, colidx, _ = random_sym_csr(rng, M, float(rng.uniform(1, 8)))
    else:  # unsymmetric pattern with diagonal entries and empty rows
        rowptr, colidx, _ = random_csr(rng, M, M, 0.04, empty_row_frac=0.2)
    parent, child_order = oracle.dendrogram(rowptr, colidx)
    lparent, lchild = literal.dendrogram(rowptr, colidx)
    assert list(parent) == lparent and list(child_order) == lchild
    for seg_len in (7, 1024):
        perm, iperm, seq, seg = oracle.ordering(rowptr, colidx, parent, child_order, seg_len, details=True)
        lperm, liperm = literal.ordering(rowptr, colidx, lparent, lchild, seg_len)
        assert list(perm) == lperm and list(iperm) == liperm
        assert sorted(perm) == list(range(M))
        # the leaves of one segment occupy one contiguous range of new ids
        for b, e in zip(seg[:-1], seg[1:]):
            assert sorted(perm[b:e]) == sorted(seq[b:e])
        flat = [v for tree in literal.leaf_sequence(lparent, lchild) for v in tree]
        assert list(seq) == flat


def test_reordering_recovers_hidden_blocks():
    """Quality, not parity: on a block model with shuffled labels the reordering must raise the
    mean number of stored entries per tile (MeanNNZTC, Section 4.3.1)."""
    import workloads as wl
    rowptr, colidx, vals = wl.sbm(2048, 64, 0.25, 4.0, 7, relabel=True)
    perm, _ = oracle.reorder(rowptr, colidx)
    t0 = len(oracle.encode(rowptr, colidx, vals, None, 16, 16)["tc_offset"]) - 1
    t1 = len(oracle.encode(rowptr, colidx, vals, perm, 16, 16)["tc_offset"]) - 1
    assert t1 < 0.6 * t0


def test_column_order_against_brute_force_and_its_defining_properties():
    rng = np.random.default_rng(5)
    for K, nnz in ((1, 0), (7, 3), (50, 400), (300, 5000)):
        # skewed use counts: squares of uniform numbers favour the low ids
        colidx = (rng.random(nnz) ** 3 * K).astype(np.int32)
        order, rank = oracle.column_order(colidx, K)
        count = [0] * K
        for c in colidx.tolist():
            count[c] += 1
        def cls(n):                      # floor(log2(n)) by integer shifts, -1 for unused columns
            k = -1
            while n:
                n >>= 1
                k += 1
            return k
        brute = sorted(range(K), key=lambda c: (-cls(count[c]), c))
        assert order.tolist() == brute
        assert sorted(order.tolist()) == list(range(K))
        assert all(rank[order[j]] == j for j in range(K))
        classes = [cls(count[c]) for c in order]
        assert classes == sorted(classes, reverse=True)


def test_column_order_keeps_inputs_with_even_counts_in_place():
    K = 64
    colidx = np.repeat(np.arange(K, dtype=np.int32), 5)      # every column used 5 times
    order, rank = oracle.column_order(colidx, K)
    assert order.tolist() == list(range(K)) and rank.tolist() == list(range(K))
