"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Tolerance for C (fp16 inputs, exact fp16 x fp16 products, fp32 accumulation in any order):
|C - C_ref| <= 2e-3 * (|A|.|B|) + 1e-5 elementwise.  Format arrays and the permutation are
compared bit for bit.
"""
import os

import numpy as np
import pytest

import oracle
import paper_2501_09251_amd as acc
import workloads as wl
from _util import csr_from_rows, random_csr, f16, bf16, bf16_to_f64

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    acc.load()


def run_spmm(plan, B_u16, M, N, naive=False):
    dev = torch.device("cuda:0")
    Bd = torch.from_numpy(B_u16.view(np.int16)).to(dev)
    # poison C: every element must be overwritten; nothing behind its last row may be
    rows, guard = max(M, 1), 4096
    buf = torch.full((rows * N + guard,), float("nan"), dtype=torch.float32, device=dev)
    buf[rows * N:] = 12345.0
    C = buf[:rows * N].view(rows, N)
    stream = torch.cuda.current_stream().cuda_stream
    (acc.acc_spmm_execute_csr_naive if naive else acc.acc_spmm_execute)(plan, Bd, N, C, stream)
    torch.cuda.synchronize()
    assert bool((buf[rows * N:] == 12345.0).all()), "wrote past the end of C"
    return C[:M].cpu().numpy()


def check_against_oracle(rowptr, colidx, vals, B, C, rows=None, value_type="f16"):
    C_ref, bound = oracle.spmm(rowptr, colidx, vals, B, rows=rows, value_type=value_type)
    got = C if rows is None else C[rows]
    ok, ratio = oracle.within_bound(got, C_ref, bound)
    assert ok, f"outside tolerance, worst error/limit = {ratio}"
    return ratio


def check_format(plan, rowptr, colidx, vals, WH=16, TW=16, operand_order=0):
    perm = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_PERM)
    rank = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_COL_RANK)
    if len(rank):                       # the plan's arrays hold columns in its own column order
        colidx, vals = sorted_rows(rowptr, rank[colidx], vals)
    fmt = oracle.encode(rowptr, colidx, vals, perm, WH, TW)
    if len(rank) and operand_order == 0:
        # B in the caller's order: the most used plan columns name rows of the gathered copy
        # (as ~p), the others the input column
        order = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_COL_ORDER)
        H = acc.acc_spmm_plan_stats(plan)["num_hot_columns"]
        a2b = fmt["sparse_a_to_b"]
        fmt["sparse_a_to_b"] = np.where(a2b < H, ~a2b, order[a2b]).astype(np.int32)
    for which, key in ((acc.ACC_SPMM_ARR_ROW_WINDOW_OFFSET, "row_window_offset"), (acc.ACC_SPMM_ARR_TC_OFFSET, "tc_offset"),
                       (acc.ACC_SPMM_ARR_SPARSE_A_TO_B, "sparse_a_to_b"), (acc.ACC_SPMM_ARR_TC_LOCAL_BIT, "tc_local_bit"),
                       (acc.ACC_SPMM_ARR_VALUES, "vals")):
        np.testing.assert_array_equal(acc.acc_spmm_plan_export(plan, which), fmt[key], err_msg=key)
    return perm, fmt


def sorted_rows(rowptr, colidx, vals):
    """Oracle input must have ascending columns; the library accepts any order."""
    ci, va = colidx.copy(), vals.copy()
    for i in range(len(rowptr) - 1):
        s = slice(rowptr[i], rowptr[i + 1])
        o = np.argsort(ci[s], kind="stable")
        ci[s], va[s] = ci[s][o], va[s][o]
    return ci, va


# ------------------------------------------------------------------ small, element by element
@pytest.mark.parametrize("cfg,shrink", [(1, 0), (2, 6), (3, 6), (4, 4), (5, 7)])
@pytest.mark.parametrize("mode", ["default", "plain"])
def test_workloads_small_full_comparison(cfg, shrink, mode):
    w = wl.config(cfg, shrink)
    opt = None if mode == "default" else acc.make_options(reorder=acc.ACC_SPMM_OFF, load_balance=acc.ACC_SPMM_OFF)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, opt)
    try:
        perm, fmt = check_format(plan, w.rowptr, w.colidx, w.vals)
        st = acc.acc_spmm_plan_stats(plan)
        assert st["num_tiles"] == len(fmt["tc_offset"]) - 1 and st["nnz"] == w.nnz
        assert abs(st["ibd"] - oracle.ibd(fmt["row_window_offset"])) < 1e-9
        if st["reorder_applied"]:
            np.testing.assert_array_equal(perm, oracle.reorder(w.rowptr, w.colidx)[0])
        else:
            np.testing.assert_array_equal(perm, np.arange(w.M))
        C = run_spmm(plan, w.B, w.M, w.N)
        check_against_oracle(w.rowptr, w.colidx, w.vals, w.B, C)
    finally:
        acc.acc_spmm_destroy(plan)


# powers of two and multiples of 128 fill whole feature slabs; the others exercise the masked
# tail with every lane width (N odd, N = 2, 4, 8 mod 16), one and two slabs per wave, and
# several waves per item
@pytest.mark.parametrize("N", [16, 32, 64, 128, 256, 384, 512, 1024,
                               1, 7, 17, 2, 30, 602, 4, 36, 100, 500, 8, 24, 40, 48, 96, 136, 200, 640])
@pytest.mark.parametrize("lb", [acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON])
def test_all_widths_with_and_without_load_balancing(N, lb):
    rng = np.random.default_rng(N + lb)
    M, K = 333, 500                                    # several windows, ragged tail (333 = 20*16 + 13)
    rowptr, colidx, vals = random_csr(rng, M, K, 0.04)
    # one heavy row so that its window is split when balancing with a small cap
    heavy = np.sort(rng.choice(K, 450, replace=False)).astype(np.int32)
    rows = [colidx[rowptr[i]:rowptr[i + 1]].tolist() for i in range(M)]
    rows[40] = heavy.tolist()
    rowptr, colidx, _ = csr_from_rows(rows)
    vals = f16(rng.uniform(-1, 1, len(colidx)))
    B = f16(rng.standard_normal((K, N)))
    plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                acc.make_options(load_balance=lb, max_tiles_per_item=8, keep_csr=1))
    try:
        st = acc.acc_spmm_plan_stats(plan)
        assert (st["num_split_windows"] >= 1) == (lb == acc.ACC_SPMM_ON)
        check_format(plan, rowptr, colidx, vals)
        C = run_spmm(plan, B, M, N)
        check_against_oracle(rowptr, colidx, vals, B, C)
        C2 = run_spmm(plan, B, M, N)
        np.testing.assert_array_equal(C, C2)          # fixed summation order: bitwise repeatable
        Cn = run_spmm(plan, B, M, N, naive=True)
        check_against_oracle(rowptr, colidx, vals, B, Cn)
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("N", [32, 128, 256, 36, 200])
@pytest.mark.parametrize("cfg,shrink", [(5, 9), (3, 7)])
def test_every_kernel_variant(N, cfg, shrink):
    """All pipeline depths (0 = no prefetch), both store policies and the three ways of fetching
    the packed values give the same, correct C; on sparse tiles (one feature slab per wave) and on
    dense ones (two)."""
    w = wl.config(cfg, shrink)
    B = wl.dense(w.K, N, 77, "normal", 0.0, 1.0)
    ref = None
    for depth in (0, 1, 2, 3):
        for streaming, fetch in ((0, 1), (1, 1), (0, 2), (1, 2), (0, 3), (1, 3)):
            opt = acc.make_options(load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=16, streaming_stores=streaming,
                                   no_prefetch=int(depth == 0), pipeline_depth=depth, value_fetch=fetch)
            plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, opt)
            try:
                C = run_spmm(plan, B, w.M, N)
            finally:
                acc.acc_spmm_destroy(plan)
            if ref is None:
                ref = C
                check_against_oracle(w.rowptr, w.colidx, w.vals, B, C)
            else:
                np.testing.assert_array_equal(C, ref)      # same summation order in every variant


@pytest.mark.parametrize("N", [32, 64, 128, 384])
def test_lds_staging_gives_the_same_result(N):
    """The comparison form of the tile kernel (B rows through an LDS double buffer, as the paper's
    Algorithm 2 stages them) against the oracle and, bit for bit, against the default form; both value
    fetches, split windows, with and without a column order (the two-matrix addressing)."""
    w = wl.config(5, 9)
    B = wl.dense(w.K, N, 78, "normal", 0.0, 1.0)
    for column_order in (acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON):
        ref = None
        for lds, fetch in ((0, 1), (1, 1), (1, 2), (0, 3), (1, 3)):
            opt = acc.make_options(load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=16, value_fetch=fetch,
                                   lds_staging=lds, column_order=column_order)
            plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, opt)
            try:
                assert acc.acc_spmm_plan_stats(plan)["num_split_windows"] > 0
                C = run_spmm(plan, B, w.M, N)
            finally:
                acc.acc_spmm_destroy(plan)
            if ref is None:
                ref = C
                check_against_oracle(w.rowptr, w.colidx, w.vals, B, C)
            else:
                np.testing.assert_array_equal(C, ref)
    # widths the comparison form does not cover are refused, not silently run another way
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, acc.make_options(lds_staging=1))
    try:
        for bad_N in (16, 100, 256):
            with pytest.raises(acc.AccSpmmError) as e:
                run_spmm(plan, wl.dense(w.K, bad_N, 1, "normal", 0.0, 1.0), w.M, bad_N)
            assert e.value.code == -3
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("fetch", [0, 1, 2, 3])
@pytest.mark.parametrize("N", [16, 64, 128, 512, 17, 50, 100, 200, 640])
def test_dense_tiles_at_odd_value_offsets(fetch, N):
    """Full 16x16 tiles whose packed values start at an odd index (a one-entry first tile),
    tiles with more than 128 and more than 254 values, and a ragged last tile: the cases that
    decide how many 64-dword chunks the cooperative value fetch reads.  Plans with dense tiles
    are also the ones whose waves take two feature slabs each: the widths cover that shape with
    and without a masked tail at every lane width."""
    rng = np.random.default_rng(N)
    rows = [[0]] + [list(range(40)) for _ in range(15)]           # window 0: 1 + 15*16, 240, 120 entries
    rows += [list(range(40)) for _ in range(16)]                  # window 1: 256, 256, 128
    rows += [list(range(0, 40, 3)) for _ in range(9)]             # window 2: ragged, sparse
    rowptr, colidx, _ = csr_from_rows(rows)
    vals = f16(rng.uniform(-1, 1, len(colidx)))
    B = f16(rng.standard_normal((40, N)))
    plan = acc.acc_spmm_plan_ex(len(rows), 40, len(colidx), rowptr, colidx, vals,
                                acc.make_options(reorder=acc.ACC_SPMM_OFF, value_fetch=fetch, keep_csr=1))
    try:
        check_format(plan, rowptr, colidx, vals)
        C = run_spmm(plan, B, len(rows), N)
        check_against_oracle(rowptr, colidx, vals, B, C)
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("N", [16, 64, 128, 256, 100, 7])
@pytest.mark.parametrize("fetch", [1, 2, 3])
def test_bfloat16_values(N, fetch):
    """value_type = bfloat16: same bits-in, fp32-out contract, wide-exponent inputs that binary16
    could not hold, split windows, and the one-row-per-wave comparison kernel."""
    rng = np.random.default_rng(1000 + N)
    M, K = 333, 500
    rowptr, colidx, _ = random_csr(rng, M, K, 0.04)
    rows = [colidx[rowptr[i]:rowptr[i + 1]].tolist() for i in range(M)]
    rows[40] = np.sort(rng.choice(K, 450, replace=False)).tolist()
    rowptr, colidx, _ = csr_from_rows(rows)
    vals = bf16(rng.uniform(-1, 1, len(colidx)) * 10.0 ** rng.integers(-8, 9, len(colidx)))
    B = bf16(rng.standard_normal((K, N)) * 1e6)
    plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                acc.make_options(load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=8, keep_csr=1,
                                                 value_type=acc.ACC_SPMM_BF16, value_fetch=fetch))
    try:
        C = run_spmm(plan, B, M, N)
        check_against_oracle(rowptr, colidx, vals, B, C, value_type="bf16")
        Cn = run_spmm(plan, B, M, N, naive=True)
        check_against_oracle(rowptr, colidx, vals, B, Cn, value_type="bf16")
        packed = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_VALUES)
        assert sorted(packed.tolist()) == sorted(vals.tolist())          # bits pass through the encoder untouched
    finally:
        acc.acc_spmm_destroy(plan)


def _permuted(plan, X, to_caller=0):
    """X (numpy, K rows) through acc_spmm_permute_rows."""
    src = torch.from_numpy(np.ascontiguousarray(X).view(np.int16 if X.dtype == np.uint16 else X.dtype)).cuda()
    dst = torch.zeros_like(src)
    acc.acc_spmm_permute_rows(plan, src, dst, X.shape[1] * X.dtype.itemsize, to_caller, None)
    torch.cuda.synchronize()
    return dst.cpu().numpy().view(X.dtype)


@pytest.mark.parametrize("cfg,shrink", [(2, 6), (5, 7), (4, 4), (1, 0)])
@pytest.mark.parametrize("operand_order", [0, 1])
def test_column_order_forced_on(cfg, shrink, operand_order):
    """The plan's column order equals its definition, the tile format is that of the relabelled
    matrix, and C is the same whether execute gathers B itself or is handed B in plan order."""
    w = wl.config(cfg, shrink)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(column_order=acc.ACC_SPMM_ON, operand_order=operand_order, keep_csr=1))
    try:
        st = acc.acc_spmm_plan_stats(plan)
        assert st["column_order_applied"] == 1
        order, rank = oracle.column_order(w.colidx, w.K)
        np.testing.assert_array_equal(acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_COL_ORDER), order)
        np.testing.assert_array_equal(acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_COL_RANK), rank)
        check_format(plan, w.rowptr, w.colidx, w.vals, operand_order=operand_order)
        assert st["num_hot_columns"] == (min(w.K // 16, 1 << 17) if operand_order == 0 else 0)
        B_plan = _permuted(plan, w.B)
        np.testing.assert_array_equal(B_plan, w.B[order])
        np.testing.assert_array_equal(_permuted(plan, B_plan, to_caller=1), w.B)
        B_given = B_plan if operand_order == 1 else w.B
        C = run_spmm(plan, B_given, w.M, w.N)
        check_against_oracle(w.rowptr, w.colidx, w.vals, w.B, C)
        Cn = run_spmm(plan, B_given, w.M, w.N, naive=True)
        check_against_oracle(w.rowptr, w.colidx, w.vals, w.B, Cn)
        for N in (7, 200):                                   # the gathered-B buffer grows with N; odd row sizes
            B2 = wl.dense(w.K, N, 5, "normal", 0.0, 1.0)
            C2 = run_spmm(plan, _permuted(plan, B2) if operand_order == 1 else B2, w.M, N)
            check_against_oracle(w.rowptr, w.colidx, w.vals, B2, C2)
    finally:
        acc.acc_spmm_destroy(plan)


def test_column_order_auto_detects_hubs_at_power_of_two_labels():
    """AUTO relabels the unscrambled R-MAT graph (its heavy columns are the ids with few set
    bits) and leaves alone the same graph under random labels, the randomly labelled block
    model, the mesh and the uniform matrix."""
    def applied(M, K, rowptr, colidx, vals):
        plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                    acc.make_options(reorder=acc.ACC_SPMM_OFF))
        try:
            st = acc.acc_spmm_plan_stats(plan)
            return st["column_order_applied"], st["hub_label_skew"]
        finally:
            acc.acc_spmm_destroy(plan)

    w = wl.config(5, 3, with_B=False)                         # 2^20 vertices
    on, skew = applied(w.M, w.K, w.rowptr, w.colidx, w.vals)
    assert on == 1 and skew >= 8.0
    relabel = np.random.default_rng(0).permutation(w.K).astype(np.int32)
    on, skew = applied(w.M, w.K, w.rowptr, relabel[w.colidx], w.vals)
    assert on == 0 and skew < 2.5
    w = wl.config(5, 5, with_B=False)                         # 2^18 vertices: same labels, but B is small
    on, skew = applied(w.M, w.K, w.rowptr, w.colidx, w.vals)
    assert on == 0 and skew >= 8.0
    for cfg, shrink in ((4, 1), (3, 3)):
        w = wl.config(cfg, shrink, with_B=False)
        assert w.K >= 65536
        on, skew = applied(w.M, w.K, w.rowptr, w.colidx, w.vals)
        assert on == 0 and skew < 2.5, (cfg, skew)
    rng = np.random.default_rng(1)
    M = K = 100000
    colidx = np.sort(rng.integers(0, K - 8, (M, 8)), axis=1) + np.arange(8)     # distinct inside a row
    rowptr = np.arange(M + 1, dtype=np.int32) * 8
    on, skew = applied(M, K, rowptr, np.ascontiguousarray(colidx.reshape(-1).astype(np.int32)),
                       f16(np.ones(M * 8)))
    assert on == 0 and skew < 2.5


# ------------------------------------------------------------------ C in 16 bits
def run_spmm_c16(plan, B_u16, M, N):
    dev = torch.device("cuda:0")
    Bd = torch.from_numpy(B_u16.view(np.int16)).to(dev)
    rows, guard = max(M, 1), 4096
    buf = torch.full((rows * N + guard,), 0x7fc1, dtype=torch.int16, device=dev)    # a NaN pattern in both types
    buf[rows * N:] = 12345
    C = buf[:rows * N].view(rows, N)
    acc.acc_spmm_execute_c16(plan, Bd, N, C, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bool((buf[rows * N:] == 12345).all()), "wrote past the end of C"
    return C[:M].cpu().numpy().view(np.uint16)


def check_c16(rowptr, colidx, vals, B, C_bits, value_type):
    """fp32 accumulation within the usual bound, then one rounding to the 16-bit type: half an
    ulp of the result (2^-11 relative for binary16, 2^-8 for bfloat16), doubled for slack; results
    below the type's normal range are compared with the absolute term only."""
    ref, bound = oracle.spmm(rowptr, colidx, vals, B, value_type=value_type)
    got = C_bits.view(np.float16).astype(np.float64) if value_type == "f16" else bf16_to_f64(C_bits)
    ulp = 2.0 ** -10 if value_type == "f16" else 2.0 ** -7
    tiny = 2.0 ** -24 if value_type == "f16" else 0.0
    lim = 2e-3 * bound + 1e-5 + ulp * np.abs(ref) + tiny
    assert np.isfinite(got).all(), "an element of C was not written"
    err = np.abs(got - ref)
    assert (err <= lim).all(), f"worst error/limit = {(err / lim).max()}"


@pytest.mark.parametrize("N", [7, 16, 40, 64, 96, 128, 256])
@pytest.mark.parametrize("value_type,lb", [("f16", acc.ACC_SPMM_OFF), ("f16", acc.ACC_SPMM_ON), ("bf16", acc.ACC_SPMM_ON)])
def test_sixteen_bit_output(N, value_type, lb):
    """acc_spmm_execute_c16: same plan, same kernels, C rounded once to the plan's 16-bit type;
    split windows (partial sums stay fp32), empty rows (zeros) and a ragged last window included."""
    rng = np.random.default_rng(1000 + N)
    M, K = 333, 500
    rowptr, colidx, vals = random_csr(rng, M, K, 0.06, empty_row_frac=0.15)
    if value_type == "bf16":
        vals = bf16(rng.uniform(-1, 1, len(colidx)))
        B = bf16(rng.normal(0, 1, (K, N)))
    else:
        B = f16(rng.normal(0, 1, (K, N)))
    opt = acc.make_options(reorder=acc.ACC_SPMM_ON, load_balance=lb, max_tiles_per_item=4,
                           value_type=acc.ACC_SPMM_BF16 if value_type == "bf16" else acc.ACC_SPMM_FP16)
    plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals, opt)
    try:
        if lb == acc.ACC_SPMM_ON:
            assert acc.acc_spmm_plan_stats(plan)["num_split_windows"] > 0
        C16 = run_spmm_c16(plan, B, M, N)
        check_c16(rowptr, colidx, vals, B, C16, value_type)
        empty = np.flatnonzero(np.diff(rowptr) == 0)
        assert len(empty) and not C16[empty].any()
        # the same call in fp32, rounded here, gives the same bits
        C32 = run_spmm(plan, B, M, N)
        expect = f16(C32) if value_type == "f16" else bf16(C32)
        np.testing.assert_array_equal(C16, expect)
    finally:
        acc.acc_spmm_destroy(plan)


def test_sixteen_bit_output_on_a_workload_with_column_order():
    w = wl.config(2, 5)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(reorder=acc.ACC_SPMM_ON, load_balance=acc.ACC_SPMM_ON,
                                                 column_order=acc.ACC_SPMM_ON, max_tiles_per_item=16))
    try:
        C16 = run_spmm_c16(plan, w.B, w.M, w.N)
        check_c16(w.rowptr, w.colidx, w.vals, w.B, C16, "f16")
        np.testing.assert_array_equal(C16, f16(run_spmm(plan, w.B, w.M, w.N)))
    finally:
        acc.acc_spmm_destroy(plan)


# ------------------------------------------------------------------ sampled dense-dense product
def run_sddmm(plan, X_u16, Y_u16, nnz, N, use_values):
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X_u16.view(np.int16)).to(dev)
    Yd = torch.from_numpy(Y_u16.view(np.int16)).to(dev)
    guard = 1024
    buf = torch.full((nnz + guard,), float("nan"), dtype=torch.float32, device=dev)   # every entry must be written
    buf[nnz:] = 12345.0
    acc.acc_spmm_sddmm(plan, Xd, Yd, N, buf, use_values, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bool((buf[nnz:] == 12345.0).all()), "wrote past the end of out"
    return buf[:nnz].cpu().numpy()


def check_sddmm(rowptr, colidx, vals, X, Y, got, use_values, value_type="f16"):
    ref, bound = oracle.sddmm(rowptr, colidx, X, Y, vals if use_values else None, value_type=value_type)
    ok, ratio = oracle.within_bound(got, ref, bound)
    assert ok, f"outside tolerance, worst error/limit = {ratio}"


@pytest.mark.parametrize("N", [32, 64, 96, 128, 256, 384, 512, 640])
@pytest.mark.parametrize("lb,use_values", [(acc.ACC_SPMM_OFF, 0), (acc.ACC_SPMM_ON, 1)])
def test_sddmm_all_widths(N, lb, use_values):
    rng = np.random.default_rng(N + lb)
    M, K = 333, 500                                    # ragged last window, a window split by the balancer,
    rowptr, colidx, _ = random_csr(rng, M, K, 0.04)    # empty rows and (rows 64..95) three empty windows in a row
    rows = [colidx[rowptr[i]:rowptr[i + 1]].tolist() for i in range(M)]
    rows[40] = np.sort(rng.choice(K, 450, replace=False)).tolist()
    for i in range(64, 112):
        rows[i] = []
    rowptr, colidx, _ = csr_from_rows(rows)
    vals = f16(rng.uniform(-1, 1, len(colidx)))
    X, Y = f16(rng.standard_normal((M, N))), f16(rng.standard_normal((K, N)))
    plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                acc.make_options(load_balance=lb, max_tiles_per_item=8, keep_entry_map=1))
    try:
        st = acc.acc_spmm_plan_stats(plan)
        assert (st["num_split_windows"] >= 1) == (lb == acc.ACC_SPMM_ON)
        got = run_sddmm(plan, X, Y, len(colidx), N, use_values)
        check_sddmm(rowptr, colidx, vals, X, Y, got, use_values)
        np.testing.assert_array_equal(got, run_sddmm(plan, X, Y, len(colidx), N, use_values))   # repeatable
        # the same plan still does SpMM
        C = run_spmm(plan, Y, M, N)
        check_against_oracle(rowptr, colidx, vals, Y, C)
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("cfg,shrink", [(2, 6), (4, 4), (3, 6), (5, 7)])
def test_sddmm_on_the_workloads_reordered(cfg, shrink):
    """Row reordering on (where AUTO takes it): out stays in the caller's entry order."""
    w = wl.config(cfg, shrink)
    X = wl.dense(w.M, 64, 3, "normal", 0.0, 1.0)
    Y = wl.dense(w.K, 64, 4, "normal", 0.0, 1.0)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(reorder=acc.ACC_SPMM_ON, keep_entry_map=1))
    try:
        got = run_sddmm(plan, X, Y, w.nnz, 64, 1)
        check_sddmm(w.rowptr, w.colidx, w.vals, X, Y, got, 1)
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("cfg,shrink", [(2, 6), (5, 7)])
def test_sddmm_with_column_order_and_Y_in_the_callers_order(cfg, shrink):
    """The most used rows of Y come from the plan's gathered copy, the others from Y in place."""
    w = wl.config(cfg, shrink)
    X = wl.dense(w.M, 128, 3, "normal", 0.0, 1.0)
    Y = wl.dense(w.K, 128, 4, "normal", 0.0, 1.0)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(column_order=acc.ACC_SPMM_ON, keep_entry_map=1))
    try:
        st = acc.acc_spmm_plan_stats(plan)
        assert st["column_order_applied"] == 1 and st["num_hot_columns"] == w.K // 16
        got = run_sddmm(plan, X, Y, w.nnz, 128, 1)
        check_sddmm(w.rowptr, w.colidx, w.vals, X, Y, got, 1)
        got = run_sddmm(plan, X[:, :64].copy(), Y[:, :64].copy(), w.nnz, 64, 0)     # narrower after wider: the copy is reused
        check_sddmm(w.rowptr, w.colidx, w.vals, X[:, :64].copy(), Y[:, :64].copy(), got, 0)
        C = run_spmm(plan, Y, w.M, 128)                                              # and SpMM shares it
        check_against_oracle(w.rowptr, w.colidx, w.vals, Y, C)
    finally:
        acc.acc_spmm_destroy(plan)


def test_sddmm_bf16_and_column_order_in_plan_order():
    rng = np.random.default_rng(5)
    w = wl.config(2, 6)
    vals = bf16(rng.uniform(-1, 1, w.nnz))
    X, Y = bf16(rng.standard_normal((w.M, 128)) * 100.0), bf16(rng.standard_normal((w.K, 128)) * 0.01)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, vals,
                                acc.make_options(value_type=acc.ACC_SPMM_BF16, keep_entry_map=1,
                                                 column_order=acc.ACC_SPMM_ON, operand_order=1))
    try:
        assert acc.acc_spmm_plan_stats(plan)["column_order_applied"] == 1
        got = run_sddmm(plan, X, _permuted(plan, Y), w.nnz, 128, 1)      # Y in the plan's order, as B would be
        check_sddmm(w.rowptr, w.colidx, vals, X, Y, got, 1, value_type="bf16")
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("reorder", [acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON])
def test_update_values_keeps_the_plan(reorder):
    """New values for the same pattern: SpMM and SDDMM afterwards use them; one attention-style
    round trip (SDDMM -> values -> SpMM) stays inside the library's order conventions."""
    rng = np.random.default_rng(77)
    w = wl.config(2, 6)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(reorder=reorder, load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=16,
                                                 keep_entry_map=1))
    try:
        new_vals = f16(rng.uniform(-2, 2, w.nnz))
        acc.acc_spmm_update_values(plan, torch.from_numpy(new_vals.view(np.int16)).cuda(), None)
        np.testing.assert_array_equal(np.sort(acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_VALUES)), np.sort(new_vals))
        C = run_spmm(plan, w.B, w.M, w.N)
        check_against_oracle(w.rowptr, w.colidx, new_vals, w.B, C)
        X, Y = wl.dense(w.M, 64, 8, "normal", 0.0, 0.3), wl.dense(w.K, 64, 9, "normal", 0.0, 0.3)
        scores = run_sddmm(plan, X, Y, w.nnz, 64, 0)                  # fp32, entry order
        check_sddmm(w.rowptr, w.colidx, None, X, Y, scores, 0)
        edge_vals = f16(np.tanh(scores))                              # any entry-wise function of the scores
        acc.acc_spmm_update_values(plan, torch.from_numpy(edge_vals.view(np.int16)).cuda(), None)
        C = run_spmm(plan, w.B, w.M, w.N)
        check_against_oracle(w.rowptr, w.colidx, edge_vals, w.B, C)
    finally:
        acc.acc_spmm_destroy(plan)


def test_sddmm_argument_errors():
    rowptr, colidx, vals = csr_from_rows([[0]])
    X = torch.zeros(1, 8192, dtype=torch.float16, device="cuda")        # large enough for every width tried
    out = torch.zeros(1, device="cuda")
    plan = acc.acc_spmm_plan(1, 1, 1, rowptr, colidx, vals)
    try:
        with pytest.raises(acc.AccSpmmError) as e:
            acc.acc_spmm_sddmm(plan, X, X, 32, out)                       # built without keep_entry_map
        assert e.value.code == -1
    finally:
        acc.acc_spmm_destroy(plan)
    plan = acc.acc_spmm_plan_ex(1, 1, 1, rowptr, colidx, vals, acc.make_options(keep_entry_map=1))
    try:
        for bad_N in (0, 48, 160, 8192):
            with pytest.raises(acc.AccSpmmError) as e:
                acc.acc_spmm_sddmm(plan, X, X, bad_N, out)
            assert e.value.code == -3
    finally:
        acc.acc_spmm_destroy(plan)


def test_identity_and_permutation_matrices_are_exact():
    rng = np.random.default_rng(0)
    n, N = 100, 64
    B = f16(rng.standard_normal((n, N)))
    p = rng.permutation(n)
    for cols in (np.arange(n), p):
        rowptr, colidx, vals = csr_from_rows([[int(c)] for c in cols], np.ones(n))
        plan = acc.acc_spmm_plan(n, n, n, rowptr, colidx, vals)
        try:
            C = run_spmm(plan, B, n, N)
            np.testing.assert_array_equal(C, B.view(np.float16).astype(np.float32)[cols])
        finally:
            acc.acc_spmm_destroy(plan)


def test_reordering_is_invisible_in_C():
    w = wl.config(4, 5)
    out = []
    for ro in (acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON):
        plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, acc.make_options(reorder=ro))
        try:
            st = acc.acc_spmm_plan_stats(plan)
            assert st["reorder_applied"] == (ro == acc.ACC_SPMM_ON)
            out.append((run_spmm(plan, w.B, w.M, w.N), st["num_tiles"]))
        finally:
            acc.acc_spmm_destroy(plan)
    for C, _ in out:
        check_against_oracle(w.rowptr, w.colidx, w.vals, w.B, C)
    assert out[1][1] < 0.7 * out[0][1]                # the hidden blocks are recovered: far fewer tiles


@pytest.mark.parametrize("seg_len", [3, 64, 1024, 3000])
def test_permutation_is_bit_exact_for_all_segment_lengths(seg_len):
    """Reordering (dendrogram rounds and ordering kernel on the GPU) against the oracle's permutation."""
    from _util import random_sym_csr
    rng = np.random.default_rng(seg_len)
    graphs = [random_sym_csr(rng, 700, 6.0)[:2], random_csr(rng, 500, 500, 0.02, empty_row_frac=0.2)[:2]]
    w = wl.config(4, 6)
    graphs.append((w.rowptr, w.colidx))
    w5 = wl.config(5, 10)            # heavy-tailed: hub rows and hub columns inside segments
    graphs.append((w5.rowptr, w5.colidx))
    for rowptr, colidx in graphs:
        M = len(rowptr) - 1
        vals = np.zeros(len(colidx), np.uint16)
        plan = acc.acc_spmm_plan_ex(M, M, len(colidx), rowptr, colidx, vals,
                                    acc.make_options(reorder=acc.ACC_SPMM_ON, segment_length=seg_len))
        try:
            perm = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_PERM)
            iperm = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_IPERM)
            parent = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_DENDROGRAM_PARENT)
            assert acc.acc_spmm_plan_stats(plan)["dendrogram_on_device"] == 1
        finally:
            acc.acc_spmm_destroy(plan)
        operm, oiperm = oracle.reorder(rowptr, colidx, seg_len)
        np.testing.assert_array_equal(parent, oracle.dendrogram(rowptr, colidx)[0])
        np.testing.assert_array_equal(perm, operm)
        np.testing.assert_array_equal(iperm, oiperm)


def _dendrogram_of(rowptr, colidx, **opt):
    M = len(rowptr) - 1
    plan = acc.acc_spmm_plan_ex(M, M, len(colidx), rowptr, colidx, np.zeros(len(colidx), np.uint16),
                                acc.make_options(reorder=acc.ACC_SPMM_ON, **opt))
    try:
        st = acc.acc_spmm_plan_stats(plan)
        return acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_DENDROGRAM_PARENT), st
    finally:
        acc.acc_spmm_destroy(plan)


def test_dendrogram_rounds_on_special_graphs():
    """Step I in rounds on the GPU against the oracle on graphs that stress the rounds: a star (all
    leaves join one hub in the same rounds), a path and a ring (every vertex depends on its
    predecessor: rounds of one vertex), a clique, two cliques joined by an edge, isolated vertices,
    a hub with more neighbours than one wavefront decides (the multi-block path), and hubs that
    are each other's neighbours."""
    from _util import csr_from_edges
    rng = np.random.default_rng(11)
    graphs = {}
    n = 5000
    graphs["star"] = csr_from_edges(n, [(0, i) for i in range(1, n)])[:2]
    graphs["path"] = csr_from_edges(600, [(i, i + 1) for i in range(599)])[:2]
    graphs["ring"] = csr_from_edges(500, [(i, (i + 1) % 500) for i in range(500)])[:2]
    graphs["clique"] = csr_from_edges(60, [(i, j) for i in range(60) for j in range(i)])[:2]
    graphs["two cliques"] = csr_from_edges(40, [(i, j) for i in range(20) for j in range(i)] +
                                           [(20 + i, 20 + j) for i in range(20) for j in range(i)] + [(0, 20)])[:2]
    graphs["isolated"] = csr_from_edges(100, [(1, 2), (50, 51)])[:2]
    hubs = [(h, int(x)) for h in range(4) for x in rng.choice(np.arange(4, 20000), 3000, replace=False)]
    hubs += [(a, b) for a in range(4) for b in range(a)]
    hubs += [(int(a), int(b)) for a, b in rng.integers(4, 20000, (30000, 2)) if a != b]
    graphs["hubs"] = csr_from_edges(20000, hubs)[:2]
    for name, (rowptr, colidx) in graphs.items():
        print(f"[dendrogram] {name}", flush=True)
        parent, st = _dendrogram_of(rowptr, colidx)
        assert st["dendrogram_on_device"] == 1 and st["dendrogram_rounds"] >= 1, name
        np.testing.assert_array_equal(parent, oracle.dendrogram(rowptr, colidx)[0], err_msg=name)
        host_parent, st = _dendrogram_of(rowptr, colidx, dendrogram_on_host=1)
        assert st["dendrogram_on_device"] == 0
        np.testing.assert_array_equal(host_parent, parent, err_msg=name)


def test_dendrogram_on_larger_special_graphs():
    """Step I against the oracle where the device form's special paths carry the load: a star of 2^20 vertices (one
    list of a million records, walked by thousands of blocks and reduced by a wavefront), hubs with long lists that
    are each other's neighbours (the per-round record budget), a few hundred hubs over many leaves, cliques on a
    ring.  Whichever form ends up running, the result is the oracle's."""
    import scipy.sparse as sp

    def csr_of(M, a, b):
        a, b = np.asarray(a, np.int64), np.asarray(b, np.int64)
        A = sp.coo_matrix((np.ones(2 * len(a), np.int8), (np.concatenate([a, b]), np.concatenate([b, a]))), shape=(M, M)).tocsr()
        A.sum_duplicates()
        A.sort_indices()
        return A.indptr.astype(np.int32), A.indices.astype(np.int32)

    rng = np.random.default_rng(7)
    graphs = {}
    n = 1 << 20
    graphs["star"] = csr_of(n, np.zeros(n - 1, np.int64), np.arange(1, n))
    h = 64
    ii, jj = np.triu_indices(h, 1)
    graphs["mutual hubs"] = csr_of(300000, np.concatenate([np.repeat(np.arange(h), 20000), ii]),
                                   np.concatenate([rng.integers(h, 300000, h * 20000), jj]))
    graphs["hubs over leaves"] = csr_of(200000, rng.integers(0, 300, 400000), rng.integers(300, 200000, 400000))
    blocks = 100
    ii, jj = np.triu_indices(40, 1)
    graphs["cliques on a ring"] = csr_of(40 * blocks, np.concatenate([ii + 40 * c for c in range(blocks)] + [np.arange(blocks) * 40]),
                                         np.concatenate([jj + 40 * c for c in range(blocks)] + [(np.arange(blocks) + 1) % blocks * 40]))
    for name, (rowptr, colidx) in graphs.items():
        print(f"[dendrogram] {name}: M={len(rowptr) - 1} entries={len(colidx)}", flush=True)
        parent, st = _dendrogram_of(rowptr, colidx)
        assert st["dendrogram_rounds"] >= 1, name
        np.testing.assert_array_equal(parent, oracle.dendrogram(rowptr, colidx)[0], err_msg=name)


def test_dendrogram_of_a_banded_matrix_falls_back_to_the_host_form():
    """A chain: every vertex's decision depends on its predecessor's, so a round commits one or two
    vertices.  The device form notices that the rest would take longer than the sequential form
    needs for the whole graph and hands over; the result is the oracle's either way."""
    M = 1 << 17
    offs = np.array([-4, -3, -2, -1, 1, 2, 3, 4])
    cols = np.arange(M, dtype=np.int64)[:, None] + offs[None, :]
    ok = (cols >= 0) & (cols < M)
    rowptr = np.zeros(M + 1, np.int32)
    np.cumsum(ok.sum(1), out=rowptr[1:])
    colidx = cols[ok].astype(np.int32)
    parent, st = _dendrogram_of(rowptr, colidx)
    assert st["dendrogram_on_device"] == 0 and st["dendrogram_rounds"] >= 256
    np.testing.assert_array_equal(parent, oracle.dendrogram(rowptr, colidx)[0])


def test_unsorted_rows_in_a_large_matrix():
    """Input rows need not be sorted; in a matrix large enough for the threaded input check, rows
    with descending columns in every thread's share give the result of the sorted matrix."""
    M, K, per_row, N = 1 << 19, 1 << 16, 9, 32
    rng = np.random.default_rng(12)
    colidx = np.sort(rng.integers(0, K // per_row, (M, per_row)) + np.arange(per_row) * (K // per_row), axis=1).astype(np.int32)
    vals = f16(rng.uniform(-1, 1, (M, per_row)))
    flipped = rng.random(M) < 0.3
    given_c, given_v = colidx.copy(), vals.copy()
    given_c[flipped] = given_c[flipped, ::-1]
    given_v[flipped] = given_v[flipped, ::-1]
    rowptr = (np.arange(M + 1, dtype=np.int64) * per_row).astype(np.int32)
    assert M * per_row >= 1 << 22 and flipped[: M // 16].any() and flipped[-M // 16:].any()
    B = f16(rng.standard_normal((K, N)))
    plan = acc.acc_spmm_plan_ex(M, K, M * per_row, rowptr, given_c.ravel(), given_v.ravel(),
                                acc.make_options(reorder=acc.ACC_SPMM_OFF))
    try:
        C = run_spmm(plan, B, M, N)
        rows = np.unique(np.concatenate([np.arange(40), np.flatnonzero(flipped)[:200], rng.integers(0, M, 300), np.arange(M - 40, M)]))
        check_against_oracle(rowptr, colidx.ravel(), vals.ravel(), B, C, rows=rows)
    finally:
        acc.acc_spmm_destroy(plan)


def test_linearity_in_B_exact_on_small_integers():
    rng = np.random.default_rng(5)
    M = K = 200
    rowptr, colidx, _ = random_csr(rng, M, K, 0.05)
    vals = f16(rng.integers(-4, 5, len(colidx)))
    B1 = rng.integers(-8, 9, (K, 32)).astype(np.float64)
    B2 = rng.integers(-8, 9, (K, 32)).astype(np.float64)
    plan = acc.acc_spmm_plan(M, K, len(colidx), rowptr, colidx, vals)
    try:
        C1, C2, C12 = (run_spmm(plan, f16(b), M, 32) for b in (B1, B2, 4 * B1 + B2))
        np.testing.assert_array_equal(C12, 4 * C1 + C2)     # all sums are small integers: exact in fp32
    finally:
        acc.acc_spmm_destroy(plan)


# ------------------------------------------------------------------------------- edge cases
def test_edge_cases():
    rng = np.random.default_rng(9)
    N = 32
    # (M, K, rows)
    cases = {
        "empty matrix rows": (5, 7, [[] for _ in range(5)]),
        "single entry": (1, 1, [[0]]),
        "fewer rows than a window": (3, 40, [[0, 39], [], [5, 6, 7]]),
        "first window empty": (40, 10, [[] for _ in range(16)] + [[i % 10] for i in range(24)]),
        "exactly one full tile": (16, 16, [list(range(16)) for _ in range(16)]),
        "17 columns: second tile padded": (16, 17, [list(range(17)) for _ in range(16)]),
        "rectangular wide": (20, 3000, [sorted(rng.choice(3000, 50, replace=False).tolist()) for _ in range(20)]),
        "rectangular tall": (300, 5, [[int(rng.integers(0, 5))] for _ in range(300)]),
        "unsorted columns": (2, 9, [[8, 0, 3], [2, 1]]),
    }
    for name, (M, K, rows) in cases.items():
        rowptr, colidx, _ = csr_from_rows(rows)
        vals = f16(rng.uniform(-1, 1, len(colidx)))
        B = f16(rng.standard_normal((K, N)))
        for lb in (acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON):
            plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                        acc.make_options(load_balance=lb, max_tiles_per_item=2, keep_csr=1))
            try:
                sci, sva = sorted_rows(rowptr, colidx, vals)
                check_format(plan, rowptr, sci, sva)
                C = run_spmm(plan, B, M, N)
                check_against_oracle(rowptr, sci, sva, B, C)
                Cn = run_spmm(plan, B, M, N, naive=True)
                check_against_oracle(rowptr, sci, sva, B, Cn)
            finally:
                acc.acc_spmm_destroy(plan)
    # M == 0
    plan = acc.acc_spmm_plan(0, 4, 0, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint16))
    acc.acc_spmm_execute(plan, torch.zeros(4, N, dtype=torch.float16, device="cuda"), N,
                         torch.zeros(1, N, device="cuda"), None)
    acc.acc_spmm_destroy(plan)


def test_wide_matrix_uses_64bit_row_offsets():
    """K >= 2^24 switches the kernel to 64-bit B row offsets; columns at both ends of the range."""
    rng = np.random.default_rng(3)
    M, K, N = 100, (1 << 24) + 64, 16
    rows = []
    for i in range(M):
        cols = set(rng.integers(0, K, 20).tolist()) | {K - 1 - i, i}
        rows.append(sorted(cols))
    rowptr, colidx, _ = csr_from_rows(rows)
    vals = f16(rng.uniform(-1, 1, len(colidx)))
    B = wl.dense(K, N, 5, "normal", 0.0, 1.0)
    for lb in (acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON):
        plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                    acc.make_options(load_balance=lb, max_tiles_per_item=4))
        try:
            check_format(plan, rowptr, colidx, vals)
            C = run_spmm(plan, B, M, N)
            check_against_oracle(rowptr, colidx, vals, B, C)
        finally:
            acc.acc_spmm_destroy(plan)


# (K, N): B of 4 GiB or more, or K >= 2^24, makes execute address rows of B with 64-bit offsets.
# The widths cover every lane width of that addressing mode: 2, 4 and 8 features per lane, one and
# two feature slabs per wavefront, whole slabs and masked tails.
@pytest.mark.parametrize("dense", [False, True])
@pytest.mark.parametrize("K,N", [((1 << 24) + 64, 30), ((1 << 24) + 64, 36), ((1 << 24) + 64, 100),
                                 ((1 << 24) + 64, 128), (1 << 23, 256), (1 << 23, 512)])
def test_wide_addressing_at_every_lane_width(K, N, dense):
    """The 64-bit row-offset variants of the tile kernel at the widths real calls use (16-byte
    lanes, two slabs per wave), with both ways of fetching the packed values, all pipeline depths,
    split windows, and columns at both ends of K; every element of C against the oracle.  dense: all
    rows of a window share their columns, so that tiles are full and waves take two slabs each."""
    rng = np.random.default_rng(N)
    M = 301
    rows = []
    shared = []
    for i in range(M):
        n = 330 if i == 37 else 24                       # one heavy row: its window is split
        if dense and i % 16 == 0:
            shared = rng.integers(0, K, 72).tolist() + [K - 1 - i, i, (K // 2) + i]
        cols = set(shared) if dense and i != 37 else set(rng.integers(0, K, n).tolist()) | {K - 1 - i, i, (K // 2) + i}
        rows.append(sorted(cols))
    rowptr, colidx, _ = csr_from_rows(rows)
    vals = f16(rng.uniform(-1, 1, len(colidx)))
    print(f"[wide] generating B {K} x {N}", flush=True)
    B = wl.dense(K, N, 5, "uniform", -1.0, 1.0)
    assert K >= (1 << 24) or B.nbytes >= (1 << 32)
    dev = torch.device("cuda:0")
    Bd = torch.from_numpy(B.view(np.int16)).to(dev)
    C_ref, bound = oracle.spmm(rowptr, colidx, vals, B)
    first = None
    for fetch in (1, 2, 3):
        for depth in (0, 1, 2, 3):
            plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                        acc.make_options(load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=4,
                                                         reorder=acc.ACC_SPMM_OFF,
                                                         value_fetch=fetch, pipeline_depth=depth,
                                                         no_prefetch=int(depth == 0),
                                                         column_order=acc.ACC_SPMM_OFF))   # B read in place
            try:
                st = acc.acc_spmm_plan_stats(plan)
                assert st["num_split_windows"] >= 1 and (st["mean_nnz_per_tile"] >= 24.0) == dense
                if first is None:
                    check_format(plan, rowptr, colidx, vals)
                buf = torch.full((M * N + 4096,), float("nan"), dtype=torch.float32, device=dev)
                buf[M * N:] = 12345.0
                C = buf[:M * N].view(M, N)
                acc.acc_spmm_execute(plan, Bd, N, C, torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                assert bool((buf[M * N:] == 12345.0).all()), "wrote past the end of C"
                got = C.cpu().numpy()
            finally:
                acc.acc_spmm_destroy(plan)
            ok, ratio = oracle.within_bound(got, C_ref, bound)
            assert ok, f"fetch {fetch} depth {depth}: outside tolerance, worst error/limit = {ratio}"
            if first is None:
                first = got
            else:
                np.testing.assert_array_equal(got, first)     # same summation order in every variant
    del Bd


def test_paper_geometry_8x8_format_and_closed_form_size():
    w = wl.config(2, 7)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(window_height=8, tile_width=8, reorder=acc.ACC_SPMM_ON))
    try:
        perm, fmt = check_format(plan, w.rowptr, w.colidx, w.vals, 8, 8)
        np.testing.assert_array_equal(perm, oracle.reorder(w.rowptr, w.colidx)[0])
        st = acc.acc_spmm_plan_stats(plan)
        # Section 3.3: (ceil(M/8) + NumTCBlock*11 + 2) * 4 bytes
        assert st["index_bytes"] == (-(-w.M // 8) + 11 * st["num_tiles"] + 2) * 4
        with pytest.raises(acc.AccSpmmError) as e:
            run_spmm(plan, w.B, w.M, w.N)
        assert e.value.code == -3
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("N", [16, 32, 64, 128, 256, 512, 1, 7, 30, 36, 100, 200, 136, 640])
@pytest.mark.parametrize("lb", [acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON])
def test_tiles_of_width_32_at_all_widths(N, lb):
    """Plans with 16 x 32 tiles (the 32-deep matrix instruction): the five arrays equal the oracle's
    encoding of that geometry and every element of C is within tolerance, for every lane width, masked
    tails, one and two slabs per wave, split windows, and dense rows whose bytes are all ones."""
    rng = np.random.default_rng(1000 + N + lb)
    M, K = 333, 700
    rowptr, colidx, vals = random_csr(rng, M, K, 0.05)
    rows = [colidx[rowptr[i]:rowptr[i + 1]].tolist() for i in range(M)]
    rows[40] = np.sort(rng.choice(K, 650, replace=False)).tolist()      # heavy: its window is split
    for i in range(96, 112):                                             # one window of full 16 x 32 tiles
        rows[i] = list(range(100, 100 + 96))
    rows[200] = []
    rowptr, colidx, _ = csr_from_rows(rows)
    vals = f16(rng.uniform(-1, 1, len(colidx)))
    B = f16(rng.standard_normal((K, N)))
    plan = acc.acc_spmm_plan_ex(M, K, len(colidx), rowptr, colidx, vals,
                                acc.make_options(tile_width=32, load_balance=lb, max_tiles_per_item=4))
    try:
        st = acc.acc_spmm_plan_stats(plan)
        assert st["tile_width"] == 32 and (st["num_split_windows"] >= 1) == (lb == acc.ACC_SPMM_ON)
        check_format(plan, rowptr, colidx, vals, 16, 32)
        C = run_spmm(plan, B, M, N)
        check_against_oracle(rowptr, colidx, vals, B, C)
        np.testing.assert_array_equal(C, run_spmm(plan, B, M, N))        # fixed summation order
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("cfg,shrink", [(2, 6), (3, 6), (4, 4), (5, 7)])
@pytest.mark.parametrize("value_type", ["f16", "bf16"])
def test_tiles_of_width_32_on_the_workloads(cfg, shrink, value_type):
    """16 x 32 tiles on shrunk workloads with the library's default decisions (reordering, column
    order, load balancing), both value types, both pipeline depths, both orders of B."""
    w = wl.config(cfg, shrink)
    vals, B = w.vals, w.B
    if value_type == "bf16":
        rng = np.random.default_rng(cfg)
        vals = bf16(rng.uniform(-1, 1, w.nnz) * 2.0 ** rng.integers(-20, 20, w.nnz))
        B = bf16(rng.standard_normal((w.K, w.N)))
    vt = acc.ACC_SPMM_BF16 if value_type == "bf16" else acc.ACC_SPMM_FP16
    for depth, column_order, operand_order in ((0, acc.ACC_SPMM_AUTO, 0), (1, acc.ACC_SPMM_ON, 0), (2, acc.ACC_SPMM_ON, 1),
                                               (2, acc.ACC_SPMM_OFF, 0)):
        if operand_order == 1 and w.M != w.K:
            continue
        plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, vals,
                                    acc.make_options(tile_width=32, value_type=vt, pipeline_depth=depth,
                                                     column_order=column_order, operand_order=operand_order))
        try:
            check_format(plan, w.rowptr, w.colidx, vals, 16, 32, operand_order)
            in_plan_order = operand_order == 1 and acc.acc_spmm_plan_stats(plan)["column_order_applied"] == 1
            C = run_spmm(plan, _permuted(plan, B) if in_plan_order else B, w.M, w.N)
            check_against_oracle(w.rowptr, w.colidx, vals, B, C, value_type=value_type)
        finally:
            acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("WH,TW", [(32, 16), (64, 16), (32, 32), (8, 16)])
def test_other_tile_geometries_build_the_oracles_format(WH, TW):
    """Window heights and tile widths the execute kernel does not run: the five arrays still equal
    the oracle's encoding of the same geometry byte for byte, the statistics count that format, and
    execute refuses the plan."""
    w = wl.config(2, 7)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(window_height=WH, tile_width=TW, reorder=acc.ACC_SPMM_ON))
    try:
        perm, fmt = check_format(plan, w.rowptr, w.colidx, w.vals, WH, TW)
        st = acc.acc_spmm_plan_stats(plan)
        T = len(fmt["tc_offset"]) - 1
        assert st["num_tiles"] == T and st["window_height"] == WH and st["tile_width"] == TW
        words = -(-WH * TW // 64)
        assert st["index_bytes"] == 4 * (-(-w.M // WH) + 1) + 4 * (T + 1) + 4 * T * TW + 8 * T * words
        tr = acc.acc_spmm_plan_traffic(plan, 128)
        assert tr["b_bytes"] == st["sum_distinct_cols"] * 128 * 2 and tr["mfma_flops"] == 2 * T * WH * TW * 128
        with pytest.raises(acc.AccSpmmError) as e:
            run_spmm(plan, w.B, w.M, w.N)
        assert e.value.code == -3
    finally:
        acc.acc_spmm_destroy(plan)


def test_execute_argument_errors():
    rowptr, colidx, vals = csr_from_rows([[0]])
    plan = acc.acc_spmm_plan(1, 1, 1, rowptr, colidx, vals)
    try:
        B = torch.zeros(1, 48, dtype=torch.float16, device="cuda")
        C = torch.zeros(1, 48, device="cuda")
        for bad_N in (0, -16, 65537):
            with pytest.raises(acc.AccSpmmError) as e:
                acc.acc_spmm_execute(plan, B, bad_N, C, None)
            assert e.value.code == -3
        with pytest.raises(acc.AccSpmmError) as e:
            acc.acc_spmm_execute(plan, B, 32, None, None)
        assert e.value.code == -1
        with pytest.raises(acc.AccSpmmError) as e:
            acc.acc_spmm_execute_csr_naive(plan, B, 32, C, None)    # built without keep_csr
        assert e.value.code == -1
    finally:
        acc.acc_spmm_destroy(plan)


def test_plan_survives_a_round_trip_through_a_file(tmp_path):
    """Save, load: every exported array and statistic is the same, and so are C, the row-per-wave
    result and the sddmm output, bit for bit."""
    w = wl.config(2, 6)
    X = wl.dense(w.M, 64, 3, "normal", 0.0, 1.0)
    opt = acc.make_options(reorder=acc.ACC_SPMM_ON, load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=16,
                           column_order=acc.ACC_SPMM_ON, keep_csr=1, keep_entry_map=1)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, opt)
    path = str(tmp_path / "plan.bin")
    try:
        acc.acc_spmm_plan_save(plan, path)
        twin = acc.acc_spmm_plan_load(path)
        try:
            assert acc.acc_spmm_plan_stats(twin) == acc.acc_spmm_plan_stats(plan)
            for which in range(11):
                np.testing.assert_array_equal(acc.acc_spmm_plan_export(twin, which), acc.acc_spmm_plan_export(plan, which))
            for N in (128, 40):                                     # gathered rows at 128, plain entries at 40
                B = wl.dense(w.K, N, 6, "normal", 0.0, 1.0)
                C = run_spmm(twin, B, w.M, N)
                np.testing.assert_array_equal(C, run_spmm(plan, B, w.M, N))
                check_against_oracle(w.rowptr, w.colidx, w.vals, B, C)
                np.testing.assert_array_equal(run_spmm(twin, B, w.M, N, naive=True), run_spmm(plan, B, w.M, N, naive=True))
            Y = wl.dense(w.K, 64, 4, "normal", 0.0, 1.0)
            np.testing.assert_array_equal(run_sddmm(twin, X, Y, w.nnz, 64, 1), run_sddmm(plan, X, Y, w.nnz, 64, 1))
        finally:
            acc.acc_spmm_destroy(twin)
    finally:
        acc.acc_spmm_destroy(plan)
    # a damaged file is refused, not trusted
    blob = open(path, "rb").read()
    for name, data in (("short.bin", blob[: len(blob) // 2]), ("magic.bin", b"XX" + blob[2:]),
                       ("version.bin", blob[:8] + b"\x09\x00\x00\x00" + blob[12:]),
                       ("flipped.bin", blob[: len(blob) // 2] + bytes([blob[len(blob) // 2] ^ 0x10]) + blob[len(blob) // 2 + 1:]),
                       ("last.bin", blob[:-1] + bytes([blob[-1] ^ 1])), ("longer.bin", blob + b"\x00")):
        bad = tmp_path / name
        bad.write_bytes(data)
        with pytest.raises(acc.AccSpmmError) as e:
            acc.acc_spmm_plan_load(str(bad))
        assert e.value.code in (-1, -3)


def test_plan_with_tiles_of_width_32_through_a_file_and_the_other_execute_calls(tmp_path):
    """A 16 x 32 plan saved and loaded gives the same C bit for bit; the entry point that allocates
    nothing and the 16-bit-C call run it too; the sampled dense-dense product refuses it."""
    w = wl.config(2, 6)
    opt = acc.make_options(tile_width=32, load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=8, column_order=acc.ACC_SPMM_ON,
                           keep_entry_map=1)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, opt)
    path = str(tmp_path / "plan32.bin")
    try:
        assert acc.acc_spmm_plan_stats(plan)["num_split_windows"] >= 1
        acc.acc_spmm_plan_save(plan, path)
        twin = acc.acc_spmm_plan_load(path)
        try:
            assert acc.acc_spmm_plan_stats(twin) == acc.acc_spmm_plan_stats(plan)
            for N in (128, 40):
                B = wl.dense(w.K, N, 6, "normal", 0.0, 1.0)
                C = run_spmm(plan, B, w.M, N)
                check_against_oracle(w.rowptr, w.colidx, w.vals, B, C)
                np.testing.assert_array_equal(run_spmm(twin, B, w.M, N), C)
                dev = torch.device("cuda:0")
                Bd = torch.from_numpy(B.view(np.int16)).to(dev)
                Cs = torch.full((w.M, N), float("nan"), dtype=torch.float32, device=dev)
                acc.acc_spmm_execute_static(twin, Bd, N, Cs, torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(Cs.cpu().numpy(), C)
                C16 = torch.zeros((w.M, N), dtype=torch.float16, device=dev)
                acc.acc_spmm_execute_c16(plan, Bd, N, C16, torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                np.testing.assert_array_equal(C16.cpu().numpy(), C.astype(np.float16))
            X = torch.zeros((w.M, 64), dtype=torch.float16, device="cuda")
            out = torch.zeros(w.nnz, dtype=torch.float32, device="cuda")
            with pytest.raises(acc.AccSpmmError) as e:
                acc.acc_spmm_sddmm(plan, X, X, 64, out, 0, None)
            assert e.value.code == -3
        finally:
            acc.acc_spmm_destroy(twin)
    finally:
        acc.acc_spmm_destroy(plan)


def test_execute_can_be_captured_in_a_hip_graph():
    """After one eager call (which allocates the plan's buffers), execute only enqueues kernels:
    captured into a graph and replayed with new contents of B, with eager work between the
    replays, it gives the eager result every time."""
    w = wl.config(2, 6)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(reorder=acc.ACC_SPMM_ON, load_balance=acc.ACC_SPMM_ON,
                                                 max_tiles_per_item=16, column_order=acc.ACC_SPMM_ON))
    try:
        dev = torch.device("cuda:0")
        B = torch.from_numpy(w.B.view(np.int16)).to(dev)
        C = torch.full((w.M, w.N), float("nan"), device=dev)
        C_eager = torch.empty_like(C)
        acc.acc_spmm_execute(plan, B, w.N, C, torch.cuda.current_stream().cuda_stream)     # allocates
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            acc.acc_spmm_execute(plan, B, w.N, C, torch.cuda.current_stream().cuda_stream)
        for rep in range(4):
            new_B = wl.dense(w.K, w.N, 100 + rep, "normal", 0.0, 1.0)
            B.copy_(torch.from_numpy(new_B.view(np.int16)).to(dev))
            C.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            acc.acc_spmm_execute(plan, B, w.N, C_eager, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert torch.equal(C, C_eager), f"replay {rep} differs from the eager call"
            check_against_oracle(w.rowptr, w.colidx, w.vals, new_B, C.cpu().numpy())
    finally:
        acc.acc_spmm_destroy(plan)


def test_plan_from_device_arrays_equals_plan_from_host_arrays():
    w = wl.config(4, 4)
    host = acc.acc_spmm_plan(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals)
    dev = acc.acc_spmm_plan_device(w.M, w.K, w.nnz, torch.from_numpy(w.rowptr).cuda(), torch.from_numpy(w.colidx).cuda(),
                                   torch.from_numpy(w.vals.view(np.int16)).cuda())
    try:
        for which in range(11):
            np.testing.assert_array_equal(acc.acc_spmm_plan_export(dev, which), acc.acc_spmm_plan_export(host, which))
        C = run_spmm(dev, w.B, w.M, w.N)
        np.testing.assert_array_equal(C, run_spmm(host, w.B, w.M, w.N))
        check_against_oracle(w.rowptr, w.colidx, w.vals, w.B, C)
    finally:
        acc.acc_spmm_destroy(host)
        acc.acc_spmm_destroy(dev)


def test_widest_rows():
    """N at the documented maximum (many slab launches along gridDim.y) and just past a slab boundary."""
    rng = np.random.default_rng(4)
    M, K = 40, 50
    rowptr, colidx, vals = random_csr(rng, M, K, 0.2)
    plan = acc.acc_spmm_plan(M, K, len(colidx), rowptr, colidx, vals)
    try:
        for N in (65536, 65535, 4104):
            B = f16(rng.standard_normal((K, N)))
            C = run_spmm(plan, B, M, N)
            check_against_oracle(rowptr, colidx, vals, B, C)
    finally:
        acc.acc_spmm_destroy(plan)


def test_plans_release_their_device_memory():
    """Two hundred plans built, run (with every lazily allocated buffer in use) and destroyed:
    free device memory ends where it started."""
    w = wl.config(2, 6)
    X = torch.from_numpy(wl.dense(w.M, 64, 1, "normal", 0.0, 1.0).view(np.int16)).cuda()
    B = torch.from_numpy(w.B.view(np.int16)).cuda()
    C = torch.empty((w.M, w.N), device="cuda")
    out = torch.empty(w.nnz, device="cuda")
    opt = acc.make_options(reorder=acc.ACC_SPMM_OFF, load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=8,
                           column_order=acc.ACC_SPMM_ON, keep_csr=1, keep_entry_map=1)

    def one():
        plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, opt)
        try:
            acc.acc_spmm_execute(plan, B, w.N, C, None)
            acc.acc_spmm_sddmm(plan, X, B[:, :64].contiguous(), 64, out, 1, None)
            torch.cuda.synchronize()
        finally:
            acc.acc_spmm_destroy(plan)

    for _ in range(3):
        one()                                   # warm up allocator pools of the runtime and of torch
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(200):
        one()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 64 << 20, f"device memory shrank by {(free0 - free1) >> 20} MiB over 200 plans"


# -------------------------------------------------- random shapes x random options
@pytest.mark.parametrize("block", range(8))
def test_randomised_shapes_and_options(block):
    """Seeded sweep over shapes (empty matrices, M != K, K below one tile, one heavy row, empty
    windows) and over every option, SpMM and SDDMM, each case against the oracle."""
    rng = np.random.default_rng(9000 + block)
    for case in range(12):
        M = int(rng.choice([0, 1, 15, 16, 17, 100, 333, 1000]))
        K = int(rng.choice([1, 5, 16, 40, 257, 1000])) if rng.random() < 0.6 else max(M, 1)
        density = float(rng.choice([0.0, 0.01, 0.05, 0.3]))
        rowptr, colidx, _ = random_csr(rng, M, K, density, empty_row_frac=float(rng.choice([0.0, 0.3, 0.9])))
        rows = [colidx[rowptr[i]:rowptr[i + 1]].tolist() for i in range(M)]
        if M > 40 and rng.random() < 0.5:
            rows[int(rng.integers(0, M))] = np.sort(rng.choice(K, min(K, 400), replace=False)).tolist()
        if M > 64 and rng.random() < 0.5:
            for i in range(16, 64):
                rows[i] = []
        rowptr, colidx, _ = csr_from_rows(rows)
        nnz = len(colidx)
        use_bf16 = bool(rng.random() < 0.3)
        to_bits = bf16 if use_bf16 else f16
        vt = "bf16" if use_bf16 else "f16"
        vals = to_bits(rng.uniform(-1, 1, nnz))
        N = int(rng.choice([1, 8, 16, 24, 32, 50, 64, 128, 136, 256]))
        B = to_bits(rng.standard_normal((K, N)))
        operand_order = int(rng.integers(0, 2))
        opt = dict(reorder=int(rng.integers(0, 3)), load_balance=int(rng.integers(0, 3)),
                   max_tiles_per_item=int(rng.choice([0, 1, 3, 8, 64])), column_order=int(rng.integers(0, 3)),
                   operand_order=operand_order, value_fetch=int(rng.integers(0, 4)),
                   pipeline_depth=int(rng.integers(0, 4)), streaming_stores=int(rng.integers(0, 2)),
                   segment_length=int(rng.choice([0, 2, 37, 4096])), keep_csr=1, keep_entry_map=1,
                   value_type=acc.ACC_SPMM_BF16 if use_bf16 else acc.ACC_SPMM_FP16,
                   slabs_per_wave=int(rng.integers(0, 3)), tile_width=int(rng.choice([0, 0, 16, 32])))
        wide_tiles = opt["tile_width"] == 32
        label = f"block {block} case {case}: M={M} K={K} nnz={nnz} N={N} {opt}"
        print(label, flush=True)
        plan = acc.acc_spmm_plan_ex(M, K, nnz, rowptr, colidx, vals, acc.make_options(**opt))
        try:
            in_plan_order = operand_order == 1 and acc.acc_spmm_plan_stats(plan)["column_order_applied"] == 1
            B_given = _permuted(plan, B) if in_plan_order and K > 0 else B
            C = run_spmm(plan, B_given, M, N)
            if M > 0:
                C_ref, bound = oracle.spmm(rowptr, colidx, vals, B, value_type=vt)
                ok, ratio = oracle.within_bound(C, C_ref, bound)
                assert ok, f"{label}: spmm outside tolerance, worst error/limit = {ratio}"
                Cn = run_spmm(plan, B_given, M, N, naive=True)
                ok, ratio = oracle.within_bound(Cn, C_ref, bound)
                assert ok, f"{label}: row-per-wave kernel outside tolerance, worst error/limit = {ratio}"
            Ns = int(rng.choice([32, 96, 128, 256]))
            X, Y = to_bits(rng.standard_normal((M, Ns))), to_bits(rng.standard_normal((K, Ns)))
            Y_given = _permuted(plan, Y) if in_plan_order and K > 0 else Y
            if wide_tiles:                      # the sampled product runs plans with 16 x 16 tiles only
                continue
            got = run_sddmm(plan, X, Y_given, nnz, Ns, 1)
            if nnz > 0:
                check_sddmm(rowptr, colidx, vals, X, Y, got, 1, value_type=vt)
        finally:
            acc.acc_spmm_destroy(plan)


# -------------------------------------------------- full size, as the benchmark launches it
ORACLE_BLOCK_ROWS = 1 << 16


def _compare_whole_output(w, C):
    """Every row of C against the oracle, in blocks of 64 K rows (two fp64 arrays of the whole C
    would not fit for the largest workload).  Returns the worst error/limit."""
    worst = 0.0
    for b in range(0, w.M, ORACLE_BLOCK_ROWS):
        rows = np.arange(b, min(b + ORACLE_BLOCK_ROWS, w.M), dtype=np.int64)
        C_ref, bound = oracle.spmm(w.rowptr, w.colidx, w.vals, w.B, rows=rows)
        ok, ratio = oracle.within_bound(C[b:b + len(rows)], C_ref, bound)
        assert ok, f"rows {b}..{b + len(rows)}: outside tolerance, worst error/limit = {ratio}"
        worst = max(worst, ratio)
        if (b // ORACLE_BLOCK_ROWS) % 16 == 0:
            print(f"[full-size] rows {b}.. ok, worst error/limit so far {worst:.3g}", flush=True)
    return worst


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_full_size_whole_output(cfg):
    """The benchmark's own launch (default options) at the benchmark's sizes: every element of C
    against the oracle, the plan's structural invariants, and, where the plan reorders and the
    oracle's reordering finishes in seconds (workloads 2 and 4), the permutation bit for bit."""
    print(f"[full-size] generating workload {cfg}", flush=True)
    w = wl.config(cfg)
    print(f"[full-size] planning {w.name}: M={w.M} nnz={w.nnz}", flush=True)
    plan = acc.acc_spmm_plan(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals)     # defaults, as bench.py
    try:
        st = acc.acc_spmm_plan_stats(plan)
        print(f"[full-size] plan: {st}", flush=True)
        perm = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_PERM)
        assert np.array_equal(np.sort(perm), np.arange(w.M))                       # a bijection
        rwo = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_ROW_WINDOW_OFFSET)
        tco = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_TC_OFFSET)
        assert rwo[-1] == st["num_tiles"] and tco[-1] == w.nnz and np.all(np.diff(tco) >= 1)
        items = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_WORK_ITEMS).reshape(-1, 4)
        assert (items[:, 3] - items[:, 2]).sum() == st["num_tiles"]
        if cfg in (2, 4):
            assert st["reorder_applied"] == 1
            print("[full-size] oracle reordering", flush=True)
            operm, oiperm = oracle.reorder(w.rowptr, w.colidx)
            np.testing.assert_array_equal(perm, operm)
            np.testing.assert_array_equal(acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_IPERM), oiperm)
            np.testing.assert_array_equal(acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_DENDROGRAM_PARENT),
                                          oracle.dendrogram(w.rowptr, w.colidx)[0])
        print("[full-size] executing", flush=True)
        C = run_spmm(plan, w.B, w.M, w.N)
        assert np.isfinite(C).all()
        ratio = _compare_whole_output(w, C)
        print(f"[full-size] all {w.M} rows within tolerance, worst error/limit = {ratio:.3g}", flush=True)
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.skipif(os.environ.get("ACC_SPMM_SKIP_LONG_TESTS") == "1",
                    reason="the oracle's reordering of the 2^23-vertex graph takes a minute and a half on one host core "
                           "(with -s it reports its progress); ACC_SPMM_SKIP_LONG_TESTS=1 leaves it out")
def test_full_size_permutation_of_the_largest_workload():
    """Workload 5 (8.4 M vertices, scores around 10^17, 8192 concurrent 1024-leaf segments): the
    plan's dendrogram and permutation against the oracle's, bit for bit."""
    w = wl.config(5, with_B=False)
    print(f"[full-size perm] planning {w.name}", flush=True)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, acc.make_options(reorder=acc.ACC_SPMM_ON))
    try:
        perm = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_PERM)
        parent = acc.acc_spmm_plan_export(plan, acc.ACC_SPMM_ARR_DENDROGRAM_PARENT)
        print(f"[full-size perm] plan: {acc.acc_spmm_plan_stats(plan)}", flush=True)
    finally:
        acc.acc_spmm_destroy(plan)
    oracle.set_progress(1 << 19)
    try:
        oparent, child_order = oracle.dendrogram(w.rowptr, w.colidx)
        print("[full-size perm] oracle dendrogram done", flush=True)
        np.testing.assert_array_equal(parent, oparent)
        operm, _ = oracle.ordering(w.rowptr, w.colidx, oparent, child_order)
        np.testing.assert_array_equal(perm, operm)
    finally:
        oracle.set_progress(0)


@pytest.mark.parametrize("cfg", [2, 5])
def test_full_size_sddmm_sampled_rows(cfg):
    """acc_spmm_sddmm at the benchmark's sizes; every entry of a sample of rows against the oracle."""
    print(f"[full-size sddmm] generating workload {cfg}", flush=True)
    w = wl.config(cfg, with_B=False)
    N = 64
    X = wl.dense(w.M, N, 21, "normal", 0.0, 1.0)
    Y = wl.dense(w.K, N, 22, "normal", 0.0, 1.0)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(reorder=acc.ACC_SPMM_OFF, keep_entry_map=1))
    try:
        print("[full-size sddmm] executing", flush=True)
        got = run_sddmm(plan, X, Y, w.nnz, N, 1)
        assert np.isfinite(got).all()
        rng = np.random.default_rng(cfg)
        deg = np.diff(w.rowptr)
        rows = np.unique(np.concatenate([rng.integers(0, w.M, 3000), np.argsort(deg)[-8:], np.arange(48),
                                         np.arange(w.M - 48, w.M)]))
        # the sampled rows as a matrix of their own (same columns), so that the oracle computes only them
        sub_len = deg[rows]
        sub_rowptr = np.concatenate([[0], np.cumsum(sub_len)]).astype(np.int32)
        pick = np.concatenate([np.arange(w.rowptr[r], w.rowptr[r + 1]) for r in rows])
        print(f"[full-size sddmm] checking {len(pick)} entries of {len(rows)} rows against the oracle", flush=True)
        ref, bound = oracle.sddmm(sub_rowptr, w.colidx[pick], X[rows], Y, w.vals[pick])
        ok, ratio = oracle.within_bound(got[pick], ref, bound)
        print(f"[full-size sddmm] worst error/limit = {ratio:.3g}", flush=True)
        assert ok
    finally:
        acc.acc_spmm_destroy(plan)


def test_binding_refuses_tensors_smaller_than_the_call_needs():
    """The C ABI takes bare addresses; the Python binding, which sees tensors, refuses a B or C too small for
    the N of the call before any kernel could read or write past their end."""
    rowptr, colidx, vals = csr_from_rows([[0, 3], [1], [2, 3]])
    plan = acc.acc_spmm_plan(3, 4, 5, rowptr, colidx, vals)
    try:
        B = torch.zeros(4, 32, dtype=torch.float16, device="cuda")
        C = torch.zeros(3, 32, device="cuda")
        acc.acc_spmm_execute(plan, B, 32, C, None)
        for call in (acc.acc_spmm_execute, acc.acc_spmm_execute_static, acc.acc_spmm_execute_timed):
            with pytest.raises(ValueError):
                call(plan, B, 128, C, None)                              # both too small for N = 128
            with pytest.raises(ValueError):
                call(plan, torch.zeros(4, 128, dtype=torch.float16, device="cuda"), 128, C, None)
        with pytest.raises(ValueError):
            acc.acc_spmm_execute_c16(plan, B, 32, torch.zeros(3, 16, dtype=torch.float16, device="cuda"), None)
        torch.cuda.synchronize()
    finally:
        acc.acc_spmm_destroy(plan)


@pytest.mark.parametrize("cfg,opt", [(2, dict(tile_width=32)), (4, dict(tile_width=32)),
                                      (2, dict(value_fetch=3, slabs_per_wave=2)), (3, dict(value_fetch=3, pipeline_depth=2))])
def test_full_size_whole_output_of_the_forced_variants(cfg, opt):
    """At the benchmark's sizes, the kernel forms that the defaults do not pick there: 16 x 32 tiles, the span
    fetch on long chains of sparse tiles with two slabs per wave, the span fetch where the cooperative one is
    the default.  Every element of C against the oracle."""
    w = wl.config(cfg)
    print(f"[full-size] {w.name} with {opt}", flush=True)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, acc.make_options(**opt))
    try:
        for N in ((w.N, 256) if cfg == 2 else (w.N,)):
            B = w.B if N == w.N else wl.dense(w.K, N, 5, "normal", 0.0, 1.0)
            C = run_spmm(plan, B, w.M, N)
            assert np.isfinite(C).all()
            w2 = wl.Workload(name=w.name, M=w.M, K=w.K, N=N, rowptr=w.rowptr, colidx=w.colidx, vals=w.vals, B=B)
            ratio = _compare_whole_output(w2, C)
            print(f"[full-size] N={N}: all {w.M} rows within tolerance, worst error/limit = {ratio:.3g}", flush=True)
    finally:
        acc.acc_spmm_destroy(plan)
