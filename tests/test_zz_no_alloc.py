"""acc_spmm_execute_static: the execute call that allocates nothing.

Its temporary device buffers (partial tiles of split row windows, gathered most used rows of B)
live in one static device array of the library, so the result must equal acc_spmm_execute's bit
for bit, call after call, also when a smaller problem follows a larger one in the same array.
"""
import numpy as np
import pytest

import oracle
import paper_2501_09251_amd as acc
import workloads as wl
from _util import csr_from_rows, random_csr, f16

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    acc.load()


def _run(fn, plan, B_u16, M, N):
    """One call of `fn` on a NaN-poisoned C with a guard band behind it."""
    dev = torch.device("cuda:0")
    Bd = torch.from_numpy(B_u16.view(np.int16)).to(dev)
    guard = 4096
    buf = torch.full((M * N + guard,), float("nan"), dtype=torch.float32, device=dev)
    buf[M * N:] = 12345.0
    C = buf[:M * N].view(M, N)
    fn(plan, Bd, N, C, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert bool((buf[M * N:] == 12345.0).all()), "wrote past the end of C"
    return C.cpu().numpy()


def _within(rowptr, colidx, vals, B, C):
    C_ref, bound = oracle.spmm(rowptr, colidx, vals, B)
    ok, ratio = oracle.within_bound(C, C_ref, bound)
    assert ok, f"outside tolerance, worst error/limit = {ratio}"


def test_static_scratch_equals_execute_on_two_calls_the_second_smaller():
    """Split windows and gathered rows of B both in use; a large call, then a smaller matrix at a
    smaller N through the same static array, then the large one again."""
    big = wl.config(2, 5)                      # power-law graph, 2^15 vertices, N = 128
    small = wl.config(5, 10)                   # heavy-tailed graph, 2^13 vertices
    opts = dict(reorder=acc.ACC_SPMM_ON, load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=16,
                column_order=acc.ACC_SPMM_ON)
    plan_big = acc.acc_spmm_plan_ex(big.M, big.K, big.nnz, big.rowptr, big.colidx, big.vals, acc.make_options(**opts))
    plan_small = acc.acc_spmm_plan_ex(small.M, small.K, small.nnz, small.rowptr, small.colidx, small.vals,
                                      acc.make_options(**opts))
    try:
        for plan in (plan_big, plan_small):
            st = acc.acc_spmm_plan_stats(plan)
            assert st["num_split_windows"] > 0 and st["num_partial_slots"] > 0 and st["num_hot_columns"] > 0
        B_small = wl.dense(small.K, 72, 11, "normal", 0.0, 1.0)       # 72: masked tail lanes as well
        calls = [(plan_big, big, big.B, big.N), (plan_small, small, B_small, 72), (plan_big, big, big.B, big.N)]
        for k, (plan, w, B, N) in enumerate(calls):
            print(f"[static] call {k}: {w.name} M={w.M} N={N}", flush=True)
            C_static = _run(acc.acc_spmm_execute_static, plan, B, w.M, N)
            C_plain = _run(acc.acc_spmm_execute, plan, B, w.M, N)
            np.testing.assert_array_equal(C_static, C_plain)
            _within(w.rowptr, w.colidx, w.vals, B, C_static)
    finally:
        acc.acc_spmm_destroy(plan_big)
        acc.acc_spmm_destroy(plan_small)


def test_static_scratch_without_split_windows_or_gather():
    rng = np.random.default_rng(3)
    rowptr, colidx, vals = random_csr(rng, 200, 300, 0.05)
    B = f16(rng.standard_normal((300, 40)))
    plan = acc.acc_spmm_plan_ex(200, 300, len(colidx), rowptr, colidx, vals,
                                acc.make_options(load_balance=acc.ACC_SPMM_OFF, column_order=acc.ACC_SPMM_OFF))
    try:
        C = _run(acc.acc_spmm_execute_static, plan, B, 200, 40)
        np.testing.assert_array_equal(C, _run(acc.acc_spmm_execute, plan, B, 200, 40))
        _within(rowptr, colidx, vals, B, C)
    finally:
        acc.acc_spmm_destroy(plan)


def test_static_scratch_refuses_what_does_not_fit():
    """One heavy row split over many one-tile items at the widest N: 29 partial tiles of 4 MiB."""
    rng = np.random.default_rng(4)
    rows = [sorted(rng.choice(500, 450, replace=False).tolist())] + [[int(i)] for i in range(40)]
    rowptr, colidx, vals = csr_from_rows(rows, rng.uniform(-1, 1, 490))
    plan = acc.acc_spmm_plan_ex(41, 500, len(colidx), rowptr, colidx, vals,
                                acc.make_options(load_balance=acc.ACC_SPMM_ON, max_tiles_per_item=1))
    try:
        slots = acc.acc_spmm_plan_stats(plan)["num_partial_slots"]
        N = 65536
        assert slots * 16 * N * 4 > acc.STATIC_SCRATCH_BYTES
        B = torch.zeros((500, N), dtype=torch.int16, device="cuda")
        C = torch.zeros((41, N), dtype=torch.float32, device="cuda")
        with pytest.raises(acc.AccSpmmError) as e:
            acc.acc_spmm_execute_static(plan, B, N, C, None)
        assert e.value.code == -3 and "static buffer holds" in str(e.value)
        # a width that fits is served by the same plan
        Bn = f16(rng.standard_normal((500, 128)))
        Cs = _run(acc.acc_spmm_execute_static, plan, Bn, 41, 128)
        np.testing.assert_array_equal(Cs, _run(acc.acc_spmm_execute, plan, Bn, 41, 128))
        _within(rowptr, colidx, vals, Bn, Cs)
    finally:
        acc.acc_spmm_destroy(plan)


def test_capture_without_a_prior_call():
    """Under stream capture acc_spmm_execute refuses to allocate (status -1, nothing enqueued),
    acc_spmm_execute_static is captured as it is; the graph replays to the eager result."""
    w = wl.config(2, 6)
    plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                acc.make_options(reorder=acc.ACC_SPMM_ON, load_balance=acc.ACC_SPMM_ON,
                                                 max_tiles_per_item=16, column_order=acc.ACC_SPMM_ON))
    try:
        dev = torch.device("cuda:0")
        B = torch.from_numpy(w.B.view(np.int16)).to(dev)
        C = torch.full((w.M, w.N), float("nan"), device=dev)
        C_eager = torch.empty_like(C)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        refused = None
        with torch.cuda.graph(graph):
            s = torch.cuda.current_stream().cuda_stream
            try:
                acc.acc_spmm_execute(plan, B, w.N, C, s)          # no call at this N before: would allocate
            except acc.AccSpmmError as ex:
                refused = ex
            acc.acc_spmm_execute_static(plan, B, w.N, C, s)
        assert refused is not None and refused.code == -1 and "captured" in str(refused)
        for rep in range(3):
            new_B = wl.dense(w.K, w.N, 200 + rep, "normal", 0.0, 1.0)
            B.copy_(torch.from_numpy(new_B.view(np.int16)).to(dev))
            C.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            acc.acc_spmm_execute(plan, B, w.N, C_eager, torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert torch.equal(C, C_eager), f"replay {rep} differs from the eager call"
            _within(w.rowptr, w.colidx, w.vals, new_B, C.cpu().numpy())
    finally:
        acc.acc_spmm_destroy(plan)
