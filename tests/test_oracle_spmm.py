"""Pins for the fp64 SpMM oracle: nothing here is derived from the oracle itself."""
import numpy as np
import pytest

import oracle
from oracle import literal
from _util import csr_from_rows, random_csr, f16, bf16, bf16_to_f64


def test_f16_decode_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    mine = np.array([oracle._load().orc_f16_to_f64(int(b)) for b in bits[::3]])
    lit = np.array([literal.f16_bits_to_float(int(b)) for b in bits[::3]])
    np.testing.assert_array_equal(mine, ref[::3])
    np.testing.assert_array_equal(lit, ref[::3])


def test_bf16_decode_matches_torch_and_the_closed_form_for_every_bit_pattern():
    import torch
    from fractions import Fraction
    bits = np.arange(65536, dtype=np.uint16)
    mine = np.array([oracle._load().orc_bf16_to_f64(int(b)) for b in bits])
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(mine, ref)                      # NaNs compare equal here
    np.testing.assert_array_equal(mine, bf16_to_f64(bits))
    for b in range(0, 65536, 97):                                 # (-1)^s 2^(e-127) (1 + f/128), exactly
        s, e, f = b >> 15, (b >> 7) & 255, b & 127
        if e == 255:
            continue
        v = Fraction(f, 128) * Fraction(2) ** -126 if e == 0 else (1 + Fraction(f, 128)) * Fraction(2) ** (e - 127)
        assert Fraction(float(mine[b])) == (-v if s else v)


def test_bf16_spmm_matches_numpy_matmul():
    rng = np.random.default_rng(7)
    M, K, N = 9, 14, 5
    mask = rng.random((M, K)) < 0.4
    a_bits = bf16(rng.uniform(-2, 2, mask.sum()))
    rows = [np.nonzero(mask[i])[0].tolist() for i in range(M)]
    rowptr, colidx, _ = csr_from_rows(rows)
    A = np.zeros((M, K))
    A[mask] = bf16_to_f64(a_bits)
    b_bits = bf16(rng.uniform(-1, 1, (K, N)))
    Bd = bf16_to_f64(b_bits)
    C, bound = oracle.spmm(rowptr, colidx, a_bits, b_bits, value_type="bf16")
    np.testing.assert_allclose(C, A @ Bd, atol=1e-13)
    np.testing.assert_allclose(bound, np.abs(A) @ np.abs(Bd), atol=1e-13)
    # the same bits read as binary16 are different numbers: the type switch is not a no-op
    C16, _ = oracle.spmm(rowptr, colidx, a_bits, b_bits)
    assert not np.allclose(C16, C)


def test_bf16_rounding_helper_is_round_to_nearest_even():
    import torch
    x = np.random.default_rng(3).standard_normal(4096).astype(np.float32)
    x[:4] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -(1.0 + 2.0 ** -8)]   # ties and a non-tie
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bf16(x), ref)


@pytest.mark.parametrize("seed", range(6))
def test_matches_dense_brute_force(seed):
    rng = np.random.default_rng(seed)
    M, K, N = rng.integers(1, 64, 3)
    rowptr, colidx, vals = random_csr(rng, M, K, 0.2)
    B = f16(rng.standard_normal((K, N)))
    C, bound = oracle.spmm(rowptr, colidx, vals, B)
    Cd, bd = literal.spmm_dense(M, K, rowptr, colidx, vals, B)
    np.testing.assert_allclose(C, Cd, rtol=0, atol=1e-12)
    np.testing.assert_allclose(bound, bd, rtol=0, atol=1e-12)


def test_matches_numpy_matmul_on_transposed_operand_shapes():
    # non-square, asymmetric: a transposed operand or swapped index would not survive this
    rng = np.random.default_rng(42)
    M, K, N = 7, 13, 5
    A = np.zeros((M, K), np.float16)
    mask = rng.random((M, K)) < 0.4
    A[mask] = rng.uniform(-2, 2, mask.sum()).astype(np.float16)
    rows = [np.nonzero(mask[i])[0].tolist() for i in range(M)]
    rowptr, colidx, vals = csr_from_rows(rows, A[mask])
    Bf = rng.uniform(-1, 1, (K, N)).astype(np.float16)
    C, bound = oracle.spmm(rowptr, colidx, vals, Bf.view(np.uint16))
    np.testing.assert_allclose(C, A.astype(np.float64) @ Bf.astype(np.float64), atol=1e-13)
    np.testing.assert_allclose(bound, np.abs(A).astype(np.float64) @ np.abs(Bf).astype(np.float64), atol=1e-13)


def test_identity_gives_B_exactly():
    rng = np.random.default_rng(1)
    n, N = 50, 8
    rowptr, colidx, vals = csr_from_rows([[i] for i in range(n)], np.ones(n))
    B = f16(rng.standard_normal((n, N)))
    C, _ = oracle.spmm(rowptr, colidx, vals, B)
    np.testing.assert_array_equal(C, B.view(np.float16).astype(np.float64))


def test_permutation_matrix_permutes_rows_of_B():
    rng = np.random.default_rng(2)
    n, N = 40, 6
    p = rng.permutation(n)
    rowptr, colidx, vals = csr_from_rows([[int(p[i])] for i in range(n)], np.ones(n))
    B = f16(rng.standard_normal((n, N)))
    C, _ = oracle.spmm(rowptr, colidx, vals, B)
    np.testing.assert_array_equal(C, B.view(np.float16).astype(np.float64)[p])


def test_all_ones_counts_row_lengths():
    rng = np.random.default_rng(3)
    rowptr, colidx, _ = random_csr(rng, 30, 40, 0.3)
    vals = f16(np.ones(len(colidx)))
    B = f16(np.ones((40, 4)))
    C, bound = oracle.spmm(rowptr, colidx, vals, B)
    expect = np.repeat(np.diff(rowptr)[:, None], 4, 1).astype(np.float64)
    np.testing.assert_array_equal(C, expect)
    np.testing.assert_array_equal(bound, expect)


def test_linearity_in_B_exact_on_small_integers():
    rng = np.random.default_rng(4)
    rowptr, colidx, _ = random_csr(rng, 20, 25, 0.3)
    vals = f16(rng.integers(-4, 5, len(colidx)))
    B1 = rng.integers(-8, 9, (25, 6)).astype(np.float64)
    B2 = rng.integers(-8, 9, (25, 6)).astype(np.float64)
    alpha = 4.0
    C1, _ = oracle.spmm(rowptr, colidx, vals, f16(B1))
    C2, _ = oracle.spmm(rowptr, colidx, vals, f16(B2))
    C12, _ = oracle.spmm(rowptr, colidx, vals, f16(alpha * B1 + B2))
    np.testing.assert_array_equal(C12, alpha * C1 + C2)


def test_row_subset_and_empty_rows():
    rng = np.random.default_rng(5)
    rowptr, colidx, vals = random_csr(rng, 30, 30, 0.2, empty_row_frac=0.3)
    B = f16(rng.standard_normal((30, 5)))
    C, bound = oracle.spmm(rowptr, colidx, vals, B)
    rows = np.array([29, 0, 7, 7, 13])
    Cs, bs = oracle.spmm(rowptr, colidx, vals, B, rows=rows)
    np.testing.assert_array_equal(Cs, C[rows])
    np.testing.assert_array_equal(bs, bound[rows])
    empty = np.nonzero(np.diff(rowptr) == 0)[0]
    assert len(empty) and not C[empty].any() and not bound[empty].any()


def test_within_bound_accepts_and_rejects():
    C_ref = np.array([[1.0, -2.0]])
    bound = np.array([[1.0, 2.0]])
    ok, _ = oracle.within_bound(np.array([[1.0 + 2e-3, -2.0]], np.float32), C_ref, bound)
    assert ok
    ok, ratio = oracle.within_bound(np.array([[1.0 + 3e-3, -2.0]], np.float32), C_ref, bound)
    assert not ok and ratio > 1
    ok, _ = oracle.within_bound(np.array([[np.nan, -2.0]], np.float32), C_ref, bound)
    assert not ok


# ------------------------------------------------------------------ sampled dense-dense product
@pytest.mark.parametrize("use_values", [False, True])
def test_sddmm_matches_masked_numpy_matmul(use_values):
    # non-square, N differs from both: a swapped operand or index cannot survive this
    rng = np.random.default_rng(11)
    M, K, N = 7, 13, 5
    mask = rng.random((M, K)) < 0.4
    rows = [np.nonzero(mask[i])[0].tolist() for i in range(M)]
    a = rng.uniform(-2, 2, int(mask.sum())).astype(np.float16)
    rowptr, colidx, vals = csr_from_rows(rows, a)
    X = rng.uniform(-1, 1, (M, N)).astype(np.float16)
    Y = rng.uniform(-1, 1, (K, N)).astype(np.float16)
    out, bound = oracle.sddmm(rowptr, colidx, X.view(np.uint16), Y.view(np.uint16), vals if use_values else None)
    full = X.astype(np.float64) @ Y.astype(np.float64).T
    mag = np.abs(X).astype(np.float64) @ np.abs(Y).astype(np.float64).T
    scale = a.astype(np.float64) if use_values else np.ones(len(a))
    np.testing.assert_allclose(out, full[mask] * scale, atol=1e-13)       # row-major order of the mask = CSR order
    np.testing.assert_allclose(bound, mag[mask] * np.abs(scale), atol=1e-13)


def test_sddmm_with_one_hot_rows_picks_single_products():
    # X[i] = e_i scaled, Y[j] = e_j scaled over N = max(M, K) features: <X_i, Y_j> = s_i t_i if i == j else 0
    n = 9
    rowptr, colidx, _ = csr_from_rows([sorted([i, (i + 1) % n]) for i in range(n)])
    s_, t_ = np.arange(1, n + 1, dtype=np.float64), np.arange(2, n + 2, dtype=np.float64)
    X, Y = np.diag(s_).astype(np.float16), np.diag(t_).astype(np.float16)
    out, _ = oracle.sddmm(rowptr, colidx, X.view(np.uint16), Y.view(np.uint16))
    expect = np.array([s_[i] * t_[i] if j == i else 0.0 for i in range(n) for j in sorted([i, (i + 1) % n])])
    np.testing.assert_array_equal(out, expect)


def test_sddmm_bf16_reads_both_operands_as_bf16():
    rng = np.random.default_rng(12)
    M, K, N = 6, 8, 4
    rowptr, colidx, _ = csr_from_rows([[int(c) for c in sorted(rng.choice(K, 3, replace=False))] for _ in range(M)])
    xb, yb = bf16(rng.standard_normal((M, N)) * 1e5), bf16(rng.standard_normal((K, N)) * 1e-5)
    out, _ = oracle.sddmm(rowptr, colidx, xb, yb, value_type="bf16")
    full = bf16_to_f64(xb) @ bf16_to_f64(yb).T
    rows = np.repeat(np.arange(M), 3)
    np.testing.assert_allclose(out, full[rows, colidx], rtol=1e-14)
