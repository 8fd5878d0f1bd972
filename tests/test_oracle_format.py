"""Pins for the tile-format oracle (paper Section 3.3)."""
import numpy as np
import pytest

import oracle
from oracle import literal
from _util import csr_from_rows, random_csr, load_golden


def _words(bits_per_tile, nw):
    out = []
    for bits in bits_per_tile:
        big = sum(1 << b for b in bits)
        out += [(big >> (64 * k)) & (2 ** 64 - 1) for k in range(nw)]
    return np.array(out, np.uint64)


def test_hand_worked_8x8_example():
    g = load_golden("format_8x8_toy.json")
    rowptr, colidx, vals = csr_from_rows(g["rows"])
    for fmt in (oracle.encode(rowptr, colidx, vals, None, 8, 8),):
        np.testing.assert_array_equal(fmt["row_window_offset"], g["row_window_offset"])
        np.testing.assert_array_equal(fmt["tc_offset"], g["tc_offset"])
        np.testing.assert_array_equal(fmt["sparse_a_to_b"], g["sparse_a_to_b"])
        np.testing.assert_array_equal(fmt["tc_local_bit"], _words(g["tile_bits"], 1))
        np.testing.assert_array_equal(fmt["vals"].view(np.float16).astype(int), g["packed_values"])
        nbytes = sum(fmt[k].nbytes for k in ("row_window_offset", "tc_offset", "sparse_a_to_b", "tc_local_bit"))
        assert nbytes == g["index_bytes_closed_form"]
    lit = literal.encode(rowptr, colidx, vals, None, 8, 8)
    assert lit["row_window_offset"] == g["row_window_offset"]
    assert lit["tc_offset"] == g["tc_offset"]
    assert lit["sparse_a_to_b"] == g["sparse_a_to_b"]
    assert lit["bitmaps"] == [sum(1 << b for b in bits) for bits in g["tile_bits"]]
    assert [int(np.uint16(v).view(np.float16)) for v in lit["vals"]] == g["packed_values"]


@pytest.mark.parametrize("WH,TW", [(8, 8), (16, 16), (16, 8), (4, 4), (32, 8)])
@pytest.mark.parametrize("seed", range(3))
def test_compiled_equals_literal_and_roundtrips(WH, TW, seed):
    rng = np.random.default_rng(100 * WH + TW + seed)
    M, K = int(rng.integers(1, 90)), int(rng.integers(1, 120))
    rowptr, colidx, vals = random_csr(rng, M, K, 0.15)
    perm = rng.permutation(M).astype(np.int32) if seed else None
    fmt = oracle.encode(rowptr, colidx, vals, perm, WH, TW)
    lit = literal.encode(rowptr, colidx, vals, perm, WH, TW)
    np.testing.assert_array_equal(fmt["row_window_offset"], lit["row_window_offset"])
    np.testing.assert_array_equal(fmt["tc_offset"], lit["tc_offset"])
    np.testing.assert_array_equal(fmt["sparse_a_to_b"], np.array(lit["sparse_a_to_b"], np.int32))
    np.testing.assert_array_equal(fmt["tc_local_bit"], np.array(literal.bitmap_words(lit["bitmaps"], WH, TW), np.uint64))
    np.testing.assert_array_equal(fmt["vals"], np.array(lit["vals"], np.uint16))
    # decode(encode(A, perm)) == permuted A, exactly (both decoders)
    p = np.arange(M) if perm is None else perm
    expect = [list(zip(colidx[rowptr[i]:rowptr[i + 1]].tolist(), vals[rowptr[i]:rowptr[i + 1]].tolist())) for i in p]
    assert literal.decode(lit, M, WH, TW) == expect
    rp, ci, va = oracle.decode(fmt)
    got = [list(zip(ci[rp[r]:rp[r + 1]].tolist(), va[rp[r]:rp[r + 1]].tolist())) for r in range(M)]
    assert got == expect


@pytest.mark.parametrize("seed", range(4))
def test_structural_invariants_and_closed_form_size(seed):
    rng = np.random.default_rng(seed)
    M, K = int(rng.integers(50, 400)), int(rng.integers(50, 400))
    rowptr, colidx, vals = random_csr(rng, M, K, 0.05)
    fmt = oracle.encode(rowptr, colidx, vals, None, 8, 8)
    T = len(fmt["tc_offset"]) - 1
    nnz = len(colidx)
    # Section 3.3: (ceil(M/8) + NumTCBlock*11 + 2) * 4 bytes for the four index arrays
    nbytes = sum(fmt[k].nbytes for k in ("row_window_offset", "tc_offset", "sparse_a_to_b", "tc_local_bit"))
    assert nbytes == (-(-M // 8) + 11 * T + 2) * 4
    pop = np.array([bin(int(w)).count("1") for w in fmt["tc_local_bit"]])
    assert pop.sum() == nnz and fmt["tc_offset"][-1] == nnz
    np.testing.assert_array_equal(np.diff(fmt["tc_offset"]), pop)
    a2b = fmt["sparse_a_to_b"].reshape(T, 8)
    rwo = fmt["row_window_offset"]
    for w in range(len(rwo) - 1):
        cols = a2b[rwo[w]:rwo[w + 1]].ravel()
        if len(cols) == 0:
            continue
        d = len(np.unique(cols))
        assert np.all(np.diff(cols[:d]) > 0) and np.all(cols[d:] == cols[d - 1])   # ascending, padded by last
        assert rwo[w + 1] - rwo[w] == -(-d // 8)
        for t in range(rwo[w], rwo[w + 1]):
            word = int(fmt["tc_local_bit"][t])
            colmask = [any(word >> (r * 8 + c) & 1 for r in range(8)) for c in range(8)]
            nvalid = min(8, d - (t - rwo[w]) * 8)
            assert all(colmask[:nvalid]) and not any(colmask[nvalid:])          # every valid column is used
            if nvalid == 8:
                assert 8 <= bin(word).count("1") <= 64                              # Section 3.3: 8..64 per full tile


def test_edge_cases_empty_matrix_empty_window_ragged_tail():
    # empty matrix
    fmt = oracle.encode(np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16), None, 16, 16)
    assert list(fmt["row_window_offset"]) == [0] and list(fmt["tc_offset"]) == [0]
    # 20 rows: window 0 entirely empty, window 1 (rows 16..19, ragged) has one entry
    rows = [[] for _ in range(20)]
    rows[17] = [5]
    rowptr, colidx, vals = csr_from_rows(rows)
    fmt = oracle.encode(rowptr, colidx, vals, None, 16, 16)
    assert list(fmt["row_window_offset"]) == [0, 0, 1]
    assert list(fmt["sparse_a_to_b"]) == [5] * 16
    assert list(fmt["tc_local_bit"]) == [1 << 16, 0, 0, 0]
    # stored zero is structural: it keeps its bit
    rowptr, colidx, vals = csr_from_rows([[3]], [0.0])
    fmt = oracle.encode(rowptr, colidx, vals, None, 8, 8)
    assert list(fmt["tc_local_bit"]) == [1] and list(fmt["tc_offset"]) == [0, 1]


def test_duplicate_column_is_rejected():
    rowptr, colidx, vals = csr_from_rows([[2, 2]])
    with pytest.raises(ValueError):
        oracle.encode(rowptr, colidx, vals, None, 8, 8)


def test_ibd_matches_direct_evaluation():
    rng = np.random.default_rng(0)
    t = rng.integers(0, 50, 200)
    rwo = np.concatenate([[0], np.cumsum(t)]).astype(np.int32)
    expect = np.abs(t - t.mean()).mean()                    # Eq. 3 written out
    assert abs(oracle.ibd(rwo) - expect) < 1e-12
    assert abs(literal.ibd(rwo) - expect) < 1e-12
    assert oracle.ibd(np.array([0, 3, 6, 9], np.int32)) == 0.0
    assert oracle.ibd(np.array([0, 0, 0, 0, 40], np.int32)) == pytest.approx(15.0)   # |0-10|*3+|40-10| over 4
