"""The synthetic input generators: determinism and the structure each recipe promises."""
import numpy as np
import pytest

import workloads as wl


def _check_csr(w):
    assert w.rowptr[0] == 0 and np.all(np.diff(w.rowptr) >= 0) and w.rowptr[-1] == len(w.colidx) == len(w.vals)
    assert w.colidx.min() >= 0 and w.colidx.max() < w.K
    for i in np.random.default_rng(0).integers(0, w.M, 200):
        c = w.colidx[w.rowptr[i]:w.rowptr[i + 1]]
        assert np.all(np.diff(c) > 0)
    assert w.B.shape == (w.K, w.N) and w.B.dtype == np.uint16


@pytest.mark.parametrize("cfg,shrink", [(1, 0), (2, 6), (3, 9), (4, 5), (5, 8)])
def test_configs_are_valid_and_deterministic(cfg, shrink):
    a, b = wl.config(cfg, shrink), wl.config(cfg, shrink)
    _check_csr(a)
    for k in ("rowptr", "colidx", "vals", "B"):
        np.testing.assert_array_equal(getattr(a, k), getattr(b, k))


def test_uniform_has_exactly_eight_per_row():
    w = wl.config(1)
    assert w.M == 4096 and w.N == 32 and np.all(np.diff(w.rowptr) == 8)
    v = w.vals.view(np.float16).astype(np.float64)
    assert -1 <= v.min() < -0.9 and 0.9 < v.max() <= 1


def test_rmat_symmetrised_pattern_is_symmetric_without_self_loops():
    w = wl.config(2, 8)
    rows = np.repeat(np.arange(w.M), np.diff(w.rowptr))
    e = set(zip(rows.tolist(), w.colidx.tolist()))
    assert all((j, i) in e for i, j in e) and not any(i == j for i, j in e)
    deg = np.diff(w.rowptr)
    assert deg.max() > 20 * deg.mean()          # heavy tail
    v = w.vals.view(np.float16)
    assert v.min() >= 0 and v.max() <= 1


def test_stencil_counts():
    w = wl.config(3, 9)                         # 16^3 grid
    n = round(w.M ** (1 / 3))
    assert n ** 3 == w.M and w.nnz == (3 * n - 2) ** 3
    diag = w.colidx == np.repeat(np.arange(w.M), np.diff(w.rowptr))
    assert diag.sum() == w.M and np.all(w.vals[diag].view(np.float16) == 26.0)


def test_sbm_blocks_are_hidden_by_relabelling():
    r0, c0, _ = wl.sbm(4096, 64, 0.25, 4.0, 3, relabel=False)
    rows = np.repeat(np.arange(4096), np.diff(r0))
    intra = (rows // 64 == c0 // 64).mean()
    assert 0.75 < intra < 0.85                  # 63*0.25 intra vs 4 inter per vertex
    r1, c1, _ = wl.sbm(4096, 64, 0.25, 4.0, 3, relabel=True)
    rows = np.repeat(np.arange(4096), np.diff(r1))
    assert (rows // 64 == c1 // 64).mean() < 0.05 and len(c1) == len(c0)


def test_dense_distributions():
    u = wl.dense(512, 64, 1, "uniform", -1, 1).view(np.float16).astype(np.float64)
    assert abs(u.mean()) < 0.02 and abs(u.std() - 3 ** -0.5) < 0.02
    g = wl.dense(512, 64, 1, "normal", 0, 1).view(np.float16).astype(np.float64)
    assert abs(g.mean()) < 0.02 and abs(g.std() - 1) < 0.02
