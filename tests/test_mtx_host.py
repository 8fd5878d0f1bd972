"""The Matrix Market reader (host code of the library, no GPU) against scipy.io.mmread,
and its fp16 / bf16 conversions against numpy / torch."""
import numpy as np
import pytest
import scipy.io
import scipy.sparse as sp
import torch

import paper_2501_09251_amd as acc


def _dense_from_csr(M, K, rowptr, colidx, vals_f64):
    return sp.csr_matrix((vals_f64, colidx, rowptr), shape=(M, K)).toarray()


def _as_f64(bits, value_type):
    if value_type == acc.ACC_SPMM_FP16:
        return bits.view(np.float16).astype(np.float64)
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def _round(x, value_type):
    if value_type == acc.ACC_SPMM_FP16:
        with np.errstate(over="ignore"):
            return np.asarray(x, np.float32).astype(np.float16).astype(np.float64)
    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


@pytest.mark.parametrize("value_type", [acc.ACC_SPMM_FP16, acc.ACC_SPMM_BF16])
@pytest.mark.parametrize("symmetry", ["general", "symmetric", "skew-symmetric"])
@pytest.mark.parametrize("field", ["real", "integer", "pattern"])
def test_reader_matches_scipy(tmp_path, field, symmetry, value_type):
    if field == "pattern" and symmetry == "skew-symmetric":
        pytest.skip("the format has no skew-symmetric pattern matrices")
    rng = np.random.default_rng(hash((field, symmetry)) & 0xffff)
    n, m = (23, 23) if symmetry != "general" else (23, 31)
    A = sp.random(n, m, density=0.15, random_state=int(rng.integers(1 << 30)), format="coo")
    if field == "integer":
        A.data = rng.integers(-50, 50, len(A.data)).astype(np.float64)
        A.data[A.data == 0] = 7
    else:
        A.data = rng.standard_normal(len(A.data)) * 10.0 ** rng.integers(-3, 4, len(A.data))
    if symmetry == "symmetric":
        A = sp.tril(A, format="coo")
    elif symmetry == "skew-symmetric":
        A = sp.tril(A, k=-1, format="coo")
    path = tmp_path / "a.mtx"
    with open(path, "w") as f:
        f.write(f"%%MatrixMarket matrix coordinate {field} {symmetry}\n% a comment\n\n{n} {m} {A.nnz}\n")
        for i, j, v in zip(A.row, A.col, A.data):
            if field == "pattern":
                f.write(f"{i + 1} {j + 1}\n")
            elif field == "integer":
                f.write(f"{i + 1} {j + 1} {int(v)}\n")
            else:
                f.write(f"{i + 1}\t{j + 1}   {float(v)!r}\n")
    ref = scipy.io.mmread(str(path)).toarray().astype(np.float64)       # mirrors the triangle itself
    M, K, rowptr, colidx, vals = acc.read_matrix_market(str(path), value_type)
    assert (M, K) == (n, m) and rowptr[0] == 0 and rowptr[-1] == len(colidx)
    for i in range(M):
        assert np.all(np.diff(colidx[rowptr[i]:rowptr[i + 1]]) > 0)     # ascending, no duplicates
    got = _dense_from_csr(M, K, rowptr, colidx, _as_f64(vals, value_type))
    np.testing.assert_array_equal(got, _round(ref, value_type))
    assert len(colidx) == np.count_nonzero(ref)                          # no explicit zeros were stored here


def test_duplicates_are_summed_and_explicit_zeros_kept(tmp_path):
    path = tmp_path / "d.mtx"
    path.write_text("%%MatrixMarket matrix coordinate real general\n3 4 5\n1 2 1.5\n3 4 0.0\n1 2 2.25\n2 1 -1\n1 1 4\n")
    M, K, rowptr, colidx, vals = acc.read_matrix_market(str(path))
    assert (M, K) == (3, 4)
    assert rowptr.tolist() == [0, 2, 3, 4] and colidx.tolist() == [0, 1, 0, 3]
    assert vals.view(np.float16).tolist() == [4.0, 3.75, -1.0, 0.0]


def test_half_conversion_is_round_to_nearest_even_over_the_whole_range(tmp_path):
    rng = np.random.default_rng(1)
    x = np.concatenate([
        (rng.standard_normal(3000) * 10.0 ** rng.integers(-9, 6, 3000)),
        [65504.0, 65519.99, 65520.0, 70000.0, -65520.0, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 1.5 * 2.0 ** -24,
         2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2047.5, 2048.5, 0.0],
    ]).astype(np.float32)
    path = tmp_path / "h.mtx"
    with open(path, "w") as f:
        f.write(f"%%MatrixMarket matrix coordinate real general\n1 {len(x)} {len(x)}\n")
        for j, v in enumerate(x):
            f.write(f"1 {j + 1} {float(v)!r}\n")
    for vt in (acc.ACC_SPMM_FP16, acc.ACC_SPMM_BF16):
        _, _, _, colidx, vals = acc.read_matrix_market(str(path), vt)
        assert colidx.tolist() == list(range(len(x)))
        np.testing.assert_array_equal(_as_f64(vals, vt), _round(x, vt))


@pytest.mark.parametrize("text,code", [
    ("%%MatrixMarket matrix array real general\n2 2\n1\n2\n3\n4\n", -3),
    ("%%MatrixMarket matrix coordinate complex general\n2 2 1\n1 1 1 0\n", -3),
    ("%%MatrixMarket matrix coordinate real hermitian\n2 2 1\n1 1 1\n", -3),
    ("%%MatrixMarket matrix coordinate real general\n2 2 1\n3 1 1.0\n", -1),
    ("%%MatrixMarket matrix coordinate real general\n2 2 2\n1 1 1.0\n", -1),
    ("%%MatrixMarket matrix coordinate real general\n2 2 1\n1 1\n", -1),
    ("hello\n", -1),
])
def test_reader_refuses_what_it_does_not_support(tmp_path, text, code):
    path = tmp_path / "bad.mtx"
    path.write_text(text)
    with pytest.raises(acc.AccSpmmError) as e:
        acc.read_matrix_market(str(path))
    assert e.value.code == code


def test_missing_file_is_an_error(tmp_path):
    with pytest.raises(acc.AccSpmmError) as e:
        acc.read_matrix_market(str(tmp_path / "nope.mtx"))
    assert e.value.code == -1
