"""GPU parity of the autograd wrapper: each product it launches (forward and backward) against the
CPU oracle, and the composition of a small attention layer against a dense fp64 computation.

Gradients leave the wrapper rounded to the 16-bit operand type, so the tolerance of the SpMM /
SDDMM tests is widened by one rounding of the result to float16: 2e-3 * bound + 1e-5 + 2^-10 |ref|
(twice the half-ulp of the type).
"""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import paper_2501_09251_amd as acc
import workloads as wl
from _util import random_csr, f16

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    acc.load()


def gnn():
    from paper_2501_09251_amd import gnn as module
    return module


def half_tensor(bits, grad=False):
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.float16)).cuda()
    return t.requires_grad_() if grad else t


def bits_of(t):
    return t.detach().cpu().contiguous().numpy().view(np.uint16)


def transposed_csr(M, K, rowptr, colidx):
    """CSR of the transpose and the position in A of each of its entries."""
    S = sp.csr_matrix((np.arange(1, len(colidx) + 1, dtype=np.int64), colidx, rowptr), shape=(M, K))
    T = S.T.tocsr()
    T.sort_indices()
    return T.indptr.astype(np.int32), T.indices.astype(np.int32), (T.data - 1).astype(np.int64)


def check_rounded(got16, ref, bound, ulp=2.0 ** -10):
    got = got16.detach().float().cpu().numpy().astype(np.float64)
    lim = 2e-3 * bound + 1e-5 + ulp * np.abs(ref)
    err = np.abs(got - ref)
    assert np.isfinite(got).all()
    assert (err <= lim).all(), f"worst error/limit = {(err / lim).max()}"


@pytest.mark.parametrize("N", [64, 128])
def test_aggregate_forward_and_both_gradients_against_the_oracle(N):
    w = wl.config(2, 6)
    B_bits = wl.dense(w.K, N, 11, "normal", 0.0, 1.0)
    R_bits = wl.dense(w.M, N, 12, "normal", 0.0, 1.0)          # dC, exactly representable in 16 bits
    g = gnn().Graph(w.M, w.K, w.rowptr, w.colidx, half_tensor(w.vals), reorder=acc.ACC_SPMM_ON,
                    load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=16)
    try:
        B = half_tensor(B_bits, grad=True)
        v = half_tensor(w.vals, grad=True)
        C = g.aggregate(B, v)
        ref, bound = oracle.spmm(w.rowptr, w.colidx, w.vals, B_bits)
        ok, ratio = oracle.within_bound(C.detach().cpu().numpy(), ref, bound)
        assert ok, ratio
        (C * half_tensor(R_bits).float()).sum().backward()
        t_rowptr, t_colidx, pos = transposed_csr(w.M, w.K, w.rowptr, w.colidx)
        ref, bound = oracle.spmm(t_rowptr, t_colidx, w.vals[pos], R_bits)          # dB = A^T.dC
        check_rounded(B.grad, ref, bound)
        ref, bound = oracle.sddmm(w.rowptr, w.colidx, R_bits, B_bits)              # d vals[p] = <dC[i_p], B[j_p]>
        check_rounded(v.grad, ref, bound)
    finally:
        g.close()


def test_edge_scores_forward_and_gradients_and_values_are_restored():
    w = wl.config(4, 5)
    N = 64
    X_bits = wl.dense(w.M, N, 21, "normal", 0.0, 1.0)
    Y_bits = wl.dense(w.K, N, 22, "normal", 0.0, 1.0)
    G_bits = wl.dense(w.nnz, 1, 23, "normal", 0.0, 1.0).reshape(-1)               # d(out)
    g = gnn().Graph(w.M, w.K, w.rowptr, w.colidx, half_tensor(w.vals), column_order=acc.ACC_SPMM_ON)
    try:
        X, Y = half_tensor(X_bits, grad=True), half_tensor(Y_bits, grad=True)
        out = g.edge_scores(X, Y)
        ref, bound = oracle.sddmm(w.rowptr, w.colidx, X_bits, Y_bits)
        ok, ratio = oracle.within_bound(out.detach().cpu().numpy(), ref, bound)
        assert ok, ratio
        (out * half_tensor(G_bits).float()).sum().backward()
        ref, bound = oracle.spmm(w.rowptr, w.colidx, G_bits, Y_bits)               # dX = (A with values G).Y
        check_rounded(X.grad, ref, bound)
        t_rowptr, t_colidx, pos = transposed_csr(w.M, w.K, w.rowptr, w.colidx)
        ref, bound = oracle.spmm(t_rowptr, t_colidx, G_bits[pos], X_bits)          # dY = (A^T with values G).X
        check_rounded(Y.grad, ref, bound)
        # the backward pass put other values into both plans; the next call uses A's own again
        B_bits = wl.dense(w.K, 32, 24, "normal", 0.0, 1.0)
        B = half_tensor(B_bits, grad=True)
        C = g.aggregate(B)
        ref, bound = oracle.spmm(w.rowptr, w.colidx, w.vals, B_bits)
        ok, ratio = oracle.within_bound(C.detach().cpu().numpy(), ref, bound)
        assert ok, ratio
        C.sum().backward()
        ones = f16(np.ones((w.M, 32)))
        ref, bound = oracle.spmm(t_rowptr, t_colidx, w.vals[pos], ones)
        check_rounded(B.grad, ref, bound)
    finally:
        g.close()


def test_values_follow_the_tensor_passed_in_and_its_in_place_changes():
    rng = np.random.default_rng(5)
    rowptr, colidx, vals = random_csr(rng, 300, 200, 0.05)
    B_bits = wl.dense(200, 32, 31, "normal", 0.0, 1.0)
    g = gnn().Graph(300, 200, rowptr, colidx, half_tensor(vals), transpose=False)
    try:
        B = half_tensor(B_bits)
        other = f16(rng.uniform(-1, 1, len(vals)))
        v = half_tensor(other)
        for expect, given in ((vals, None), (other, v), (vals, None), (other, v)):
            C = g.aggregate(B, given)
            ref, bound = oracle.spmm(rowptr, colidx, expect, B_bits)
            ok, ratio = oracle.within_bound(C.cpu().numpy(), ref, bound)
            assert ok, ratio
        v.mul_(2.0)                                             # exact in binary16
        C = g.aggregate(B, v)
        ref, bound = oracle.spmm(rowptr, colidx, bits_of(v), B_bits)
        ok, ratio = oracle.within_bound(C.cpu().numpy(), ref, bound)
        assert ok, ratio
        with pytest.raises(RuntimeError):                       # no transpose: no gradient for B
            Bg = half_tensor(B_bits, grad=True)
            g.aggregate(Bg).sum().backward()
        with pytest.raises(ValueError):
            g.aggregate(B.float())
        with pytest.raises(ValueError):
            g.aggregate(B[:100])
    finally:
        g.close()


@pytest.mark.parametrize("dtype", ["float16", "bfloat16"])
def test_attention_layer_gradients_against_a_dense_fp64_computation(dtype):
    """scores = sddmm(X, Y); a = sigmoid(scores); C = A(a).B; loss = <C, R>: every gradient of the
    chain against the same chain on dense fp64 tensors (same 16-bit inputs; the wrapper rounds
    intermediate gradients to 16 bits, hence the loose tolerance)."""
    dt = getattr(torch, dtype)
    tol = 2e-2 if dtype == "float16" else 1e-1
    rng = np.random.default_rng(9)
    M, K, N = 96, 80, 32
    rowptr, colidx, _ = random_csr(rng, M, K, 0.1, empty_row_frac=0.05)
    nnz = len(colidx)
    rows = np.repeat(np.arange(M), np.diff(rowptr))
    X = torch.from_numpy(rng.normal(0, 0.5, (M, N))).to(dt).cuda().requires_grad_()
    Y = torch.from_numpy(rng.normal(0, 0.5, (K, N))).to(dt).cuda().requires_grad_()
    B = torch.from_numpy(rng.normal(0, 1.0, (K, N))).to(dt).cuda().requires_grad_()
    R = torch.from_numpy(rng.normal(0, 1.0, (M, N))).cuda()
    g = gnn().Graph(M, K, rowptr, colidx, torch.ones(nnz, dtype=dt))
    try:
        a = torch.sigmoid(g.edge_scores(X, Y)).to(dt)
        C = g.aggregate(B, a)
        (C.double() * R).sum().backward()
    finally:
        g.close()
    Xd, Yd, Bd = (t.detach().double().requires_grad_() for t in (X, Y, B))
    ri, ci = torch.from_numpy(rows).cuda(), torch.from_numpy(colidx.astype(np.int64)).cuda()
    scores = (Xd[ri] * Yd[ci]).sum(1)
    A = torch.zeros((M, K), dtype=torch.float64, device="cuda").index_put((ri, ci), torch.sigmoid(scores))
    C_ref = A @ Bd
    (C_ref * R).sum().backward()
    assert float((C.detach().double() - C_ref.detach()).abs().max()) <= tol * float(C_ref.detach().abs().max())
    for name, got, ref in (("X", X.grad, Xd.grad), ("Y", Y.grad, Yd.grad), ("B", B.grad, Bd.grad)):
        err = float((got.double() - ref).abs().max())
        assert err <= tol * float(ref.abs().max()), (name, err, float(ref.abs().max()))


def test_narrow_aggregate_is_the_rounded_fp32_one():
    w = wl.config(2, 6)
    g = gnn().Graph(w.M, w.K, w.rowptr, w.colidx, half_tensor(w.vals))
    try:
        B = half_tensor(wl.dense(w.K, 64, 61, "normal", 0.0, 1.0), grad=True)
        C32 = g.aggregate(B)
        C16 = g.aggregate(B, narrow=True)
        assert C16.dtype == torch.float16 and torch.equal(C16, C32.half())
        C16.float().sum().backward()                           # the tape runs through the narrow output too
        assert B.grad is not None and B.grad.dtype == torch.float16 and bool(torch.isfinite(B.grad).all())
    finally:
        g.close()


def test_graph_conv_module_trains_one_step():
    w = wl.config(3, 6)
    g = gnn().Graph(w.M, w.K, w.rowptr, w.colidx, half_tensor(w.vals))
    try:
        torch.manual_seed(0)
        layer = gnn().GraphConv(g, 64, 32)
        H = half_tensor(wl.dense(w.K, 64, 41, "normal", 0.0, 1.0))
        out = layer(H)
        assert out.shape == (w.M, 32) and out.dtype == torch.float32
        HW_bits = bits_of(layer.linear(H))
        ref, bound = oracle.spmm(w.rowptr, w.colidx, w.vals, HW_bits)
        ok, ratio = oracle.within_bound(out.detach().cpu().numpy(), ref, bound)
        assert ok, ratio
        out.square().mean().backward()
        assert layer.linear.weight.grad is not None and bool(torch.isfinite(layer.linear.weight.grad).all())
        assert float(layer.linear.weight.grad.abs().max()) > 0
        assert float(layer.bias.grad.abs().max()) > 0
    finally:
        g.close()


def test_rectangular_and_empty_graphs():
    rng = np.random.default_rng(17)
    M, K, N = 120, 70, 32
    rowptr, colidx, vals = random_csr(rng, M, K, 0.08, empty_row_frac=0.2)
    B_bits = wl.dense(K, N, 51, "normal", 0.0, 1.0)
    R_bits = wl.dense(M, N, 52, "normal", 0.0, 1.0)
    g = gnn().Graph(M, K, rowptr, colidx, half_tensor(vals))
    try:
        B = half_tensor(B_bits, grad=True)
        C = g.aggregate(B)
        assert C.shape == (M, N)
        ref, bound = oracle.spmm(rowptr, colidx, vals, B_bits)
        ok, ratio = oracle.within_bound(C.detach().cpu().numpy(), ref, bound)
        assert ok, ratio
        (C * half_tensor(R_bits).float()).sum().backward()
        t_rowptr, t_colidx, pos = transposed_csr(M, K, rowptr, colidx)
        ref, bound = oracle.spmm(t_rowptr, t_colidx, vals[pos], R_bits)
        assert B.grad.shape == (K, N)
        check_rounded(B.grad, ref, bound)
    finally:
        g.close()
    # no stored entries at all: C is zero and so is the gradient
    empty = gnn().Graph(M, K, np.zeros(M + 1, np.int32), np.zeros(0, np.int32), torch.zeros(0, dtype=torch.float16))
    try:
        B = half_tensor(B_bits, grad=True)
        C = empty.aggregate(B)
        assert C.shape == (M, N) and float(C.detach().abs().max()) == 0.0
        C.sum().backward()
        assert float(B.grad.abs().max()) == 0.0
    finally:
        empty.close()
