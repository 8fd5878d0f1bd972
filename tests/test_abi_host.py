"""CPU-only checks of the library: it loads, exports what the header declares, mirrors the
header's structs, validates its input, fails loudly without a GPU, and its two host stages
(reordering, schedule) agree with the oracle."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

import oracle
import paper_2501_09251_amd as acc
import workloads as wl
from _util import csr_from_rows, csr_from_edges, random_sym_csr, random_csr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "acc_spmm.h")


def _has_gpu():
    n = ctypes.c_int(0)
    try:
        hip = ctypes.CDLL("libamdhip64.so")
        return hip.hipGetDeviceCount(ctypes.byref(n)) == 0 and n.value > 0
    except OSError:
        return False


def test_library_exports_every_declared_symbol():
    text = open(HEADER).read()
    declared = set(re.findall(r"ACC_SPMM_API\s+[\w\*\s]+?\b(acc_spmm_\w+)\s*\(", text))
    assert declared == set(acc.EXPORTED_SYMBOLS)
    L = acc.load()
    for name in declared:
        assert hasattr(L, name), name


def test_ctypes_structs_mirror_the_header(tmp_path):
    fields_o = [f for f, _ in acc.acc_spmm_options._fields_]
    fields_s = [f for f, _ in acc.acc_spmm_stats._fields_]
    prog = ['#include <stdio.h>', '#include <stddef.h>', '#include "acc_spmm.h"', 'int main(void){',
            'printf("%zu %zu\\n", sizeof(acc_spmm_options), sizeof(acc_spmm_stats));']
    prog += [f'printf("%zu\\n", offsetof(acc_spmm_options, {f}));' for f in fields_o]
    prog += [f'printf("%zu\\n", offsetof(acc_spmm_stats, {f}));' for f in fields_s]
    prog += ['return 0;}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(prog))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    out = subprocess.check_output([str(exe)]).decode().split()
    assert int(out[0]) == ctypes.sizeof(acc.acc_spmm_options) and int(out[1]) == ctypes.sizeof(acc.acc_spmm_stats)
    offs = [int(x) for x in out[2:]]
    assert offs[:len(fields_o)] == [getattr(acc.acc_spmm_options, f).offset for f in fields_o]
    assert offs[len(fields_o):] == [getattr(acc.acc_spmm_stats, f).offset for f in fields_s]


def _plan_error(M, K, rowptr, colidx, vals, **opt):
    with pytest.raises(acc.AccSpmmError) as e:
        h = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals, acc.make_options(**opt) if opt else None)
        acc.acc_spmm_destroy(h)
        raise AssertionError("plan unexpectedly succeeded")
    return e.value.code


def test_invalid_input_is_reported_not_crashed():
    v = lambda n: np.zeros(n, np.uint16)
    assert _plan_error(2, 4, [0, 2, 1], [0, 1], v(2)) == -2            # rowptr decreases
    assert _plan_error(2, 4, [0, 1, 1], [0, 1], v(2)) == -2            # rowptr[M] != nnz
    assert _plan_error(2, 4, [0, 1, 2], [0, 4], v(2)) == -2            # column out of range
    assert _plan_error(2, 4, [0, 1, 2], [0, -1], v(2)) == -2
    assert _plan_error(1, 4, [0, 3], [2, 0, 2], v(3)) == -2            # duplicate column (unsorted row)
    assert _plan_error(1, 4, [1, 1], [], v(0)) == -2                   # rowptr[0] != 0
    assert _plan_error(1, 4, [0, 1], [0], v(1), window_height=12, tile_width=16) == -3
    assert _plan_error(1, 4, [0, 1], [0], v(1), reorder=7) == -1
    for bad in (dict(value_fetch=4), dict(value_fetch=-1), dict(slabs_per_wave=3), dict(slabs_per_wave=-1), dict(lds_staging=2),
                dict(column_order=3), dict(operand_order=2), dict(max_tiles_per_item=-1), dict(segment_length=-5)):
        assert _plan_error(1, 4, [0, 1], [0], v(1), **bad) == -1, bad
    for bad in (dict(tile_width=12), dict(window_height=16, tile_width=64), dict(window_height=128)):
        assert _plan_error(1, 4, [0, 1], [0], v(1), **bad) == -3, bad
    bad = acc.make_options()
    bad.struct_size = 3
    with pytest.raises(acc.AccSpmmError) as e:
        acc.acc_spmm_plan_ex(1, 4, 1, [0, 1], [0], v(1), bad)
    assert e.value.code == -1
    code, msg = acc.acc_spmm_last_error()
    assert code == -1 and "struct_size" in msg
    # a forced reordering of a matrix with 2^30 or more entries is refused before any array is read
    # (its pattern graph is indexed with 32 bits), so tiny placeholder arrays are enough here
    L = acc.load()
    one = np.zeros(4, np.int32)
    for nnz, expect in ((1 << 30, -3), ((1 << 31) - 1, -3)):
        h = L.acc_spmm_plan_ex(1 << 20, 1 << 20, nnz, one.ctypes.data, one.ctypes.data, one.ctypes.data,
                               ctypes.byref(acc.make_options(reorder=acc.ACC_SPMM_ON)))
        assert not h
        code, msg = acc.acc_spmm_last_error()
        assert code == expect and "2^30" in msg


def test_invalid_input_in_a_large_matrix_names_the_first_offence():
    """Matrices of 2^22 entries or more are checked by several threads, each over a share of the rows:
    the error still names the lowest offending entry, and a duplicate is found wherever it sits."""
    M, K, per_row = 1 << 19, 1 << 20, 10
    rng = np.random.default_rng(4)
    cols = np.sort(rng.choice(K, per_row, replace=False)).astype(np.int32)
    colidx = np.tile(cols, M)
    rowptr = (np.arange(M + 1, dtype=np.int64) * per_row).astype(np.int32)
    vals = np.zeros(len(colidx), np.uint16)
    assert len(colidx) >= 1 << 22
    for where in (17, len(colidx) // 2 + 3, len(colidx) - 5):
        bad = colidx.copy()
        bad[where] = K
        bad[len(colidx) - 1] = -7                                   # a later offence must not be the one reported
        assert _plan_error(M, K, rowptr, bad, vals) == -2
        assert f"entry {where}" in acc.acc_spmm_last_error()[1]
    for row in (0, M // 3, M - 1):
        dup = colidx.copy()
        dup[row * per_row + 4] = dup[row * per_row + 3]
        assert _plan_error(M, K, rowptr, dup, vals) == -2
        assert f"in row {row}" in acc.acc_spmm_last_error()[1]


@pytest.mark.skipif(_has_gpu(), reason="only meaningful on a machine without a GPU")
def test_no_gpu_means_a_loud_error_not_a_fallback():
    code = _plan_error(2, 2, [0, 1, 2], [0, 1], np.zeros(2, np.uint16))
    assert code == -5 and "no HIP device" in acc.acc_spmm_last_error()[1]


# --------------------------------------------------------------- host stage: dendrogram
def _pattern_graph(rowptr, colidx):
    """Symmetric adjacency of A + A^T without the diagonal, built with scipy (independent of
    both the library and the oracle)."""
    import scipy.sparse as sp
    M = len(rowptr) - 1
    A = sp.csr_matrix((np.ones(len(colidx), np.int8), colidx, rowptr), shape=(M, M))
    G = ((A + A.T) != 0).astype(np.int8).tolil()
    G.setdiag(0)
    G = G.tocsr()
    G.eliminate_zeros()
    G.sort_indices()
    return G.indptr.astype(np.int64), G.indices.astype(np.int32)


def _check_dendrogram(rowptr, colidx, seg):
    M = len(rowptr) - 1
    gptr, gadj = _pattern_graph(rowptr, colidx)
    parent, seq, seg_start, work = acc.acc_spmm_dendrogram_host(M, gptr, gadj, seg)
    oparent, ochild = oracle.dendrogram(rowptr, colidx)
    np.testing.assert_array_equal(parent, oparent)
    _, _, oseq, oseg = oracle.ordering(rowptr, colidx, oparent, ochild, seg, details=True)
    np.testing.assert_array_equal(seq, oseq)
    np.testing.assert_array_equal(seg_start, oseg)
    assert work >= 1.0 or M == 0
    return parent


@pytest.mark.parametrize("seed", range(6))
def test_dendrogram_host_equals_oracle_on_random_graphs(seed):
    rng = np.random.default_rng(seed)
    M = int(rng.integers(30, 400))
    if seed % 2:
        rowptr, colidx, _ = random_sym_csr(rng, M, float(rng.uniform(1, 10)))
    else:
        rowptr, colidx, _ = random_csr(rng, M, M, 0.03, empty_row_frac=0.2)
    for seg in (5, 64, 1024):
        _check_dendrogram(rowptr, colidx, seg)


@pytest.mark.parametrize("cfg,shrink", [(1, 0), (2, 5), (3, 6), (4, 3), (5, 8)])
def test_dendrogram_host_equals_oracle_on_the_workloads(cfg, shrink):
    w = wl.config(cfg, shrink, with_B=False)
    _check_dendrogram(w.rowptr, w.colidx, 1024)


def test_dendrogram_host_special_graphs_and_bad_input():
    for M, edges in ((12, [(0, i) for i in range(1, 12)]), (5, []), (9, [(i, i + 1) for i in range(8)])):
        rowptr, colidx, _ = csr_from_edges(M, edges)
        _check_dendrogram(rowptr, colidx, 4)
    for gptr, gadj in (([0, 1, 2], [0, 0]),       # self loop
                       ([0, 2, 2], [1, 1]),       # not ascending
                       ([0, 1, 2], [1, 5])):      # out of range
        with pytest.raises(acc.AccSpmmError) as e:
            acc.acc_spmm_dendrogram_host(2, gptr, gadj)
        assert e.value.code == -2


# ----------------------------------------------------------------- host stage: schedule
def _check_schedule(rwo, items, cap, balanced, slots):
    W = len(rwo) - 1
    covered_w = np.zeros(W, np.int32)
    tiles = np.zeros(int(rwo[-1]), np.int32)
    seen_slots = []
    for w0, w1, t0, t1 in items.tolist():
        if w1 < 0:                                   # slice of a heavy window
            assert rwo[w0] <= t0 < t1 <= rwo[w0 + 1] and t1 - t0 <= cap
            assert rwo[w0 + 1] - rwo[w0] > cap
            seen_slots.append(-w1 - 1)
        else:                                        # run of whole windows
            assert 0 <= w0 < w1 <= W and t0 == rwo[w0] and t1 == rwo[w1]
            covered_w[w0:w1] += 1
            if balanced:
                assert t1 - t0 <= cap or w1 - w0 == 1
        tiles[t0:t1] += 1
    assert np.all(tiles == 1)                        # every tile exactly once
    heavy = np.diff(rwo) > cap if balanced else np.zeros(W, bool)
    assert np.all(covered_w[~heavy] == 1) and np.all(covered_w[heavy] == 0)   # every window written once
    assert sorted(seen_slots) == list(range(slots))


@pytest.mark.parametrize("seed", range(5))
def test_schedule_partitions_tiles_and_windows(seed):
    rng = np.random.default_rng(seed)
    W = int(rng.integers(1, 300))
    t = rng.integers(0, 12, W)
    t[rng.integers(0, W, 3)] = rng.integers(100, 2000, 3)     # a few heavy windows
    t[rng.integers(0, W, 10)] = 0                             # and empty ones
    rwo = np.concatenate([[0], np.cumsum(t)]).astype(np.int32)
    expect_ibd = np.abs(t - t.mean()).mean()                  # Eq. 3, written out
    for cap in (16, 64):
        items, ibd, slots = acc.acc_spmm_schedule_host(rwo, acc.ACC_SPMM_ON, cap)
        assert abs(ibd - expect_ibd) < 1e-9
        _check_schedule(rwo, items, cap, True, slots)
    items, _, slots = acc.acc_spmm_schedule_host(rwo, acc.ACC_SPMM_OFF, 16)
    assert len(items) == W and slots == 0
    _check_schedule(rwo, items, 16, False, 0)


def test_schedule_auto_follows_the_ibd_threshold():
    flat = np.arange(0, 101 * 5, 5, dtype=np.int32)            # every window has 5 tiles: IBD = 0
    items, ibd, _ = acc.acc_spmm_schedule_host(flat, acc.ACC_SPMM_AUTO, 64)
    assert ibd == 0 and len(items) == 100                      # not applied: one item per window
    t = np.array([0] * 99 + [4000])
    skew = np.concatenate([[0], np.cumsum(t)]).astype(np.int32)
    items, ibd, slots = acc.acc_spmm_schedule_host(skew, acc.ACC_SPMM_AUTO, 64)
    assert ibd > 8 and slots == -(-4000 // 64)
    items2, _, _ = acc.acc_spmm_schedule_host(skew, acc.ACC_SPMM_AUTO, 64, ibd_threshold=1e9)
    assert len(items2) == 100


def test_plan_load_refuses_files_that_are_not_plans(tmp_path):
    bad = tmp_path / "x.bin"
    bad.write_bytes(b"not a plan at all, just some bytes that are long enough to hold a header")
    with pytest.raises(acc.AccSpmmError) as e:
        acc.acc_spmm_plan_load(str(bad))
    assert e.value.code == -1
    with pytest.raises(acc.AccSpmmError) as e:
        acc.acc_spmm_plan_load(str(tmp_path / "missing.bin"))
    assert e.value.code == -1


def test_autograd_wrapper_has_no_cpu_path():
    """Without a GPU the wrapper refuses to build a Graph (it never computes on the host), and it
    checks its arguments before touching the library."""
    torch = pytest.importorskip("torch")
    from paper_2501_09251_amd import gnn
    vals = torch.ones(2, dtype=torch.float16)
    if not torch.cuda.is_available():
        with pytest.raises(RuntimeError, match="needs a GPU"):
            gnn.Graph(2, 2, np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32), vals)
    else:
        with pytest.raises(TypeError):
            gnn.Graph(2, 2, np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32), vals.float())
        with pytest.raises(ValueError):
            gnn.Graph(3, 2, np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32), vals)
