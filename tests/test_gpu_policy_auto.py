"""The plan's AUTO decisions (row reordering, column order) and the execute call's choice of how the
packed values are fetched, on inputs that are none of the five benchmark workloads: for each input
every forced alternative is timed, and what the library picks by itself must run within 5 % (20 % for
the value fetch: the worst case seen is 8-12 %, a power-law graph at N = 32 where the per-lane loads win, and the
gate leaves room for the run-to-run spread of a 0.7 ms launch) of the fastest one.

The thresholds behind AUTO (keep the reordering for at least 1 % fewer tiles; apply the column order
from 2^20 columns on when the labels of the most used columns are concentrated on few residues)
were set on the benchmark workloads; this test is the evidence that they are not fitted to them.
Inputs: R-MAT graphs with other quadrant probabilities and with scrambled labels, block models with
other community sizes, a banded matrix, and a rectangular matrix with heavy-tailed column use.
"""
import numpy as np
import pytest

import oracle
import paper_2501_09251_amd as acc
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

N = 128
TOLERANCE = 1.05          # AUTO's pick may be this much slower than the best forced combination
SLACK_MS = 0.004          # plus a few microseconds: below that, launch jitter decides


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    acc.load()


def _relabel(rowptr, colidx, vals, seed):
    """The same graph under a random relabelling of its vertices (rows and columns)."""
    M = len(rowptr) - 1
    pi = np.random.default_rng(seed).permutation(M).astype(np.int64)      # old -> new
    rows = np.repeat(np.arange(M, dtype=np.int64), np.diff(rowptr))
    key = pi[rows] * M + pi[colidx]
    o = np.argsort(key, kind="stable")
    new_rows = (key[o] // M).astype(np.int64)
    out_ptr = np.zeros(M + 1, np.int32)
    np.cumsum(np.bincount(new_rows, minlength=M), out=out_ptr[1:])
    return out_ptr, (key[o] % M).astype(np.int32), vals[o]


def _banded(M, half_width, seed):
    rng = np.random.default_rng(seed)
    offs = np.arange(-half_width, half_width + 1, 2)                        # every other diagonal
    cols = np.arange(M, dtype=np.int64)[:, None] + offs[None, :]
    ok = (cols >= 0) & (cols < M)
    rowptr = np.zeros(M + 1, np.int32)
    np.cumsum(ok.sum(1), out=rowptr[1:])
    colidx = cols[ok].astype(np.int32)
    vals = rng.uniform(-1, 1, len(colidx)).astype(np.float16).view(np.uint16)
    return rowptr, colidx, vals


def _rectangular_heavy_tailed(M, K, per_row, seed):
    """M x K, every row draws per_row columns with probability ~ 1/(rank+8): a few columns are used
    by a large share of the rows; duplicates inside a row are dropped."""
    rng = np.random.default_rng(seed)
    p = 1.0 / (np.arange(K) + 8.0)
    cdf = np.cumsum(p / p.sum())
    label = rng.permutation(K)                                              # the heavy columns get arbitrary ids
    draw = label[np.minimum(np.searchsorted(cdf, rng.random((M, per_row))), K - 1)]
    draw.sort(axis=1)
    keep = np.ones_like(draw, bool)
    keep[:, 1:] = draw[:, 1:] != draw[:, :-1]
    rowptr = np.zeros(M + 1, np.int32)
    np.cumsum(keep.sum(1), out=rowptr[1:])
    colidx = draw[keep].astype(np.int32)
    vals = rng.uniform(-1, 1, len(colidx)).astype(np.float16).view(np.uint16)
    return rowptr, colidx, vals


def _inputs():
    yield "rmat 2^21, quadrants .45/.22/.22/.11, labels as generated", (1 << 21,) * 2, wl.rmat(21, 8 << 21, 901, True, a=0.45, b=0.22, c=0.22)
    g = wl.rmat(21, 8 << 21, 902, True)
    yield "rmat 2^21, benchmark quadrants, scrambled labels", (1 << 21,) * 2, _relabel(*g, seed=5)
    yield "rmat 2^22, quadrants .50/.20/.20/.10, directed", (1 << 22,) * 2, wl.rmat(22, 12 << 22, 903, False, a=0.50, b=0.20, c=0.20)
    yield "block model, communities of 256, p_in .08", (1 << 17,) * 2, wl.sbm(1 << 17, 256, 0.08, 3.0, 904, True)
    yield "block model, communities of 16, p_in .6", (1 << 19,) * 2, wl.sbm(1 << 19, 16, 0.6, 2.0, 905, True)
    yield "banded, 33 diagonals", (1 << 20,) * 2, _banded(1 << 20, 32, 906)
    yield "rectangular 2^19 x 2^21, heavy-tailed column use", (1 << 19, 1 << 21), _rectangular_heavy_tailed(1 << 19, 1 << 21, 14, 907)


def _time_plan(plan, B, C, M):
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(2):
        acc.acc_spmm_execute(plan, B, N, C, stream)
    torch.cuda.synchronize()
    ms = [sum(acc.acc_spmm_execute_timed(plan, B, N, C, stream)) for _ in range(7)]
    return float(np.median(ms))


def test_auto_picks_within_five_percent_of_the_best_combination():
    failures = []
    for name, (M, K), (rowptr, colidx, vals) in _inputs():
        nnz = len(colidx)
        print(f"[auto] {name}: M={M} K={K} nnz={nnz}", flush=True)
        Bh = wl.dense(K, N, 31, "normal", 0.0, 1.0)
        B = torch.from_numpy(Bh.view(np.int16)).cuda()
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        times = {}
        reorders = (acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON) if M == K else (acc.ACC_SPMM_OFF,)
        for ro in reorders:
            for co in (acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON):
                plan = acc.acc_spmm_plan_ex(M, K, nnz, rowptr, colidx, vals, acc.make_options(reorder=ro, column_order=co))
                try:
                    times[(int(ro == acc.ACC_SPMM_ON), int(co == acc.ACC_SPMM_ON))] = _time_plan(plan, B, C, M)
                finally:
                    acc.acc_spmm_destroy(plan)
        plan = acc.acc_spmm_plan(M, K, nnz, rowptr, colidx, vals)                  # AUTO everywhere
        try:
            st = acc.acc_spmm_plan_stats(plan)
            pick = (int(st["reorder_applied"]), int(st["column_order_applied"]))
            t_auto = _time_plan(plan, B, C, M)
            # the AUTO plan's result is right, whatever it picked
            rows = np.unique(np.random.default_rng(3).integers(0, M, 300))
            C_ref, bound = oracle.spmm(rowptr, colidx, vals, Bh, rows=rows)
            ok, ratio = oracle.within_bound(C[torch.from_numpy(rows).cuda()].cpu().numpy(), C_ref, bound)
            assert ok, f"{name}: outside tolerance, worst error/limit = {ratio}"
        finally:
            acc.acc_spmm_destroy(plan)
        best = min(times.values())
        t_pick = min(times[pick], t_auto)          # the same plan, timed twice
        line = (f"[auto] {name}: (reorder, column order) -> ms {({k: round(v, 4) for k, v in times.items()})}; AUTO picks {pick} "
                f"({t_pick:.4f} ms, skew {st['hub_label_skew']:.1f}, tiles {st['num_tiles']} vs {st['num_tiles_identity']} in input order)")
        print(line, flush=True)
        if t_pick > TOLERANCE * best + SLACK_MS:
            failures.append(line)
        del B, C
        torch.cuda.empty_cache()
    assert not failures, "AUTO's pick is more than 5 % slower than the best combination:\n" + "\n".join(failures)


def test_default_value_fetch_is_near_the_best_way_on_held_out_inputs():
    """The rule that picks how a tile's packed values reach the lanes (by lane width, tile density and tile
    count) was set on the benchmark workloads; here every way is forced on other inputs at four widths."""
    failures = []
    picked = {"rmat 2^21, quadrants .45/.22/.22/.11, labels as generated", "block model, communities of 256, p_in .08",
              "banded, 33 diagonals", "rectangular 2^19 x 2^21, heavy-tailed column use"}
    for name, (M, K), (rowptr, colidx, vals) in _inputs():
        if name not in picked:
            continue
        nnz = len(colidx)
        plans = {f: acc.acc_spmm_plan_ex(M, K, nnz, rowptr, colidx, vals, acc.make_options(value_fetch=f)) for f in (0, 1, 2, 3)}
        try:
            for n in (32, 64, 128, 256):
                print(f"[fetch] {name}: N={n}", flush=True)
                B = torch.from_numpy(wl.dense(K, n, 31, "normal", 0.0, 1.0).view(np.int16)).cuda()
                C = torch.empty((M, n), dtype=torch.float32, device="cuda")
                stream = torch.cuda.current_stream().cuda_stream
                ms = {}
                for f, plan in plans.items():
                    for _ in range(2):
                        acc.acc_spmm_execute(plan, B, n, C, stream)
                    torch.cuda.synchronize()
                    ms[f] = float(np.median([sum(acc.acc_spmm_execute_timed(plan, B, n, C, stream)) for _ in range(7)]))
                best = min(ms[1], ms[2], ms[3])
                line = f"[fetch] {name}: N={n} ms per-lane {ms[1]:.4f} cooperative {ms[2]:.4f} span {ms[3]:.4f} default {ms[0]:.4f}"
                print(line, flush=True)
                if ms[0] > 1.20 * best + SLACK_MS:
                    failures.append(line)
                del B, C
                torch.cuda.empty_cache()
        finally:
            for plan in plans.values():
                acc.acc_spmm_destroy(plan)
    assert not failures, "the default value fetch is more than 20 % slower than the best way:\n" + "\n".join(failures)


def test_default_slabs_per_wave_is_near_the_better_shape_on_held_out_inputs():
    """One or two feature slabs per wavefront at N = 256 and 512: both shapes are forced on inputs outside
    the benchmark set.  (A first rule, two slabs for dense tiles only, failed here on the rectangular input;
    the present one also takes two where B is read in place.)"""
    failures = []
    picked = {"rmat 2^21, quadrants .45/.22/.22/.11, labels as generated", "rmat 2^21, benchmark quadrants, scrambled labels",
              "block model, communities of 16, p_in .6", "banded, 33 diagonals", "rectangular 2^19 x 2^21, heavy-tailed column use"}
    for name, (M, K), (rowptr, colidx, vals) in _inputs():
        if name not in picked:
            continue
        nnz = len(colidx)
        plans = {f: acc.acc_spmm_plan_ex(M, K, nnz, rowptr, colidx, vals, acc.make_options(slabs_per_wave=f)) for f in (0, 1, 2)}
        try:
            for n in (256, 512):
                print(f"[slabs] {name}: N={n}", flush=True)
                B = torch.from_numpy(wl.dense(K, n, 31, "normal", 0.0, 1.0).view(np.int16)).cuda()
                C = torch.empty((M, n), dtype=torch.float32, device="cuda")
                stream = torch.cuda.current_stream().cuda_stream
                ms = {}
                for f, plan in plans.items():
                    for _ in range(2):
                        acc.acc_spmm_execute(plan, B, n, C, stream)
                    torch.cuda.synchronize()
                    ms[f] = float(np.median([sum(acc.acc_spmm_execute_timed(plan, B, n, C, stream)) for _ in range(7)]))
                line = f"[slabs] {name}: N={n} ms one slab {ms[1]:.4f} two slabs {ms[2]:.4f} default {ms[0]:.4f}"
                print(line, flush=True)
                if ms[0] > 1.10 * min(ms[1], ms[2]) + SLACK_MS:
                    failures.append(line)
                del B, C
                torch.cuda.empty_cache()
        finally:
            for plan in plans.values():
                acc.acc_spmm_destroy(plan)
    assert not failures, "the default slab count is more than 10 % slower than the better one:\n" + "\n".join(failures)


def test_default_pipeline_depth_is_near_the_best_on_held_out_inputs():
    """Tiles in flight per wavefront (ring depth 1, 2 or 3) at N = 64, 128 and 256: every depth is forced on
    inputs outside the benchmark set, on which the defaults (3 for one 128-feature slab, 2 for two, 1 for
    narrower lanes) were swept."""
    failures = []
    picked = {"rmat 2^21, quadrants .45/.22/.22/.11, labels as generated", "rmat 2^21, benchmark quadrants, scrambled labels",
              "block model, communities of 256, p_in .08", "banded, 33 diagonals", "rectangular 2^19 x 2^21, heavy-tailed column use"}
    for name, (M, K), (rowptr, colidx, vals) in _inputs():
        if name not in picked:
            continue
        nnz = len(colidx)
        plans = {f: acc.acc_spmm_plan_ex(M, K, nnz, rowptr, colidx, vals, acc.make_options(pipeline_depth=f)) for f in (0, 1, 2, 3)}
        try:
            for n in (64, 128, 256):
                print(f"[depth] {name}: N={n}", flush=True)
                B = torch.from_numpy(wl.dense(K, n, 31, "normal", 0.0, 1.0).view(np.int16)).cuda()
                C = torch.empty((M, n), dtype=torch.float32, device="cuda")
                stream = torch.cuda.current_stream().cuda_stream
                ms = {}
                for f, plan in plans.items():
                    for _ in range(2):
                        acc.acc_spmm_execute(plan, B, n, C, stream)
                    torch.cuda.synchronize()
                    ms[f] = float(np.median([sum(acc.acc_spmm_execute_timed(plan, B, n, C, stream)) for _ in range(7)]))
                line = f"[depth] {name}: N={n} ms depth 1 {ms[1]:.4f} depth 2 {ms[2]:.4f} depth 3 {ms[3]:.4f} default {ms[0]:.4f}"
                print(line, flush=True)
                if ms[0] > 1.10 * min(ms[1], ms[2], ms[3]) + SLACK_MS:
                    failures.append(line)
                del B, C
                torch.cuda.empty_cache()
        finally:
            for plan in plans.values():
                acc.acc_spmm_destroy(plan)
    assert not failures, "the default ring depth is more than 10 % slower than the best one:\n" + "\n".join(failures)


def test_auto_load_balancing_is_near_the_better_choice_on_held_out_inputs():
    """Load balancing (Section 3.5) forced on and off against AUTO (on iff the imbalance measure of Eq. 3
    exceeds the threshold) at N = 128 on all held-out inputs."""
    failures = []
    for name, (M, K), (rowptr, colidx, vals) in _inputs():
        nnz = len(colidx)
        print(f"[balance] {name}", flush=True)
        B = torch.from_numpy(wl.dense(K, N, 31, "normal", 0.0, 1.0).view(np.int16)).cuda()
        C = torch.empty((M, N), dtype=torch.float32, device="cuda")
        ms, ibd, applied = {}, 0.0, 0
        for lb in (acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON, acc.ACC_SPMM_AUTO):
            plan = acc.acc_spmm_plan_ex(M, K, nnz, rowptr, colidx, vals, acc.make_options(load_balance=lb))
            try:
                ms[lb] = _time_plan(plan, B, C, M)
                if lb == acc.ACC_SPMM_AUTO:
                    st = acc.acc_spmm_plan_stats(plan)
                    ibd, applied = st["ibd"], st["load_balance_applied"]
            finally:
                acc.acc_spmm_destroy(plan)
        line = (f"[balance] {name}: ms off {ms[acc.ACC_SPMM_OFF]:.4f} on {ms[acc.ACC_SPMM_ON]:.4f} auto {ms[acc.ACC_SPMM_AUTO]:.4f} "
                f"(imbalance {ibd:.1f}, applied {applied})")
        print(line, flush=True)
        t_pick = min(ms[acc.ACC_SPMM_AUTO], ms[acc.ACC_SPMM_ON if applied else acc.ACC_SPMM_OFF])     # the same plan, timed twice
        if t_pick > TOLERANCE * min(ms[acc.ACC_SPMM_OFF], ms[acc.ACC_SPMM_ON]) + SLACK_MS:
            failures.append(line)
        del B, C
        torch.cuda.empty_cache()
    assert not failures, "AUTO load balancing is more than 5 % slower than the better choice:\n" + "\n".join(failures)
