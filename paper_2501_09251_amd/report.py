"""Ablation and format report for one workload, in the structure of the paper's detailed
evaluation (Section 4.3): reordering quality (MeanNNZTC, 4.3.1), index footprint of the
bitmap format against CSR and an int8-per-entry tile format (4.3.2), pipeline on/off
(4.3.3), load balancing on/off (4.3.4) and the switch-by-switch ablation (4.3.5).

    python -m paper_2501_09251_amd.report --config 2
    python -m paper_2501_09251_amd.report --config 2 --variants --widths 32,64,128,256

Needs a GPU.  Prints one JSON object per line; every timing is the whole execute (gather of B
where the plan has a column order, tile kernel, split-window combine kernel), from HIP events,
averaged over --steps launches.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--shrink", type=int, default=0)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--plan-only", action="store_true",
                    help="build one plan with the row reordering forced on and print its statistics and phase times "
                         "(for profiling the preprocessing kernels); nothing is executed")
    ap.add_argument("--dendrogram-on-host", action="store_true", help="with --plan-only: the host form of Step I")
    ap.add_argument("--variants", action="store_true",
                    help="time the forms of the tile kernel that execute chooses among (value fetch, slabs per wave, ring "
                         "depth, 16x32 tiles, LDS staging) against the library's own choice, at the widths of --widths")
    ap.add_argument("--widths", default="32,64,128,256", help="with --variants: comma-separated N")
    args = ap.parse_args()

    import torch
    import paper_2501_09251_amd as acc
    import workloads as wl

    if not torch.cuda.is_available():
        print("report: no GPU visible", file=sys.stderr)
        return 2
    if args.plan_only:
        w = wl.config(args.config, args.shrink, with_B=False)
        plan = acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals,
                                    acc.make_options(reorder=acc.ACC_SPMM_ON, dendrogram_on_host=int(args.dendrogram_on_host)))
        st = acc.acc_spmm_plan_stats(plan)
        acc.acc_spmm_destroy(plan)
        print(json.dumps({"report": "plan", "workload": w.name, **{k: st[k] for k in (
            "t_total_s", "t_validate_s", "t_reorder_s", "t_graph_s", "t_dendrogram_s", "t_ordering_s", "t_column_order_s",
            "t_encode_s", "t_schedule_s", "dendrogram_on_device", "dendrogram_rounds", "reorder_work_ratio", "num_tiles",
            "num_tiles_identity")}}), flush=True)
        return 0
    if args.variants:
        return variants(args, torch, acc, wl)
    w = wl.config(args.config, args.shrink)
    dev = torch.device("cuda:0")
    B = torch.from_numpy(w.B.view(np.int16)).to(dev)
    C = torch.empty((w.M, w.N), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    OFF, ON = acc.ACC_SPMM_OFF, acc.ACC_SPMM_ON

    def plan_with(**kw):
        return acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, acc.make_options(**kw))

    def timed(**kw):
        plan = plan_with(**kw)
        try:
            st = acc.acc_spmm_plan_stats(plan)
            for _ in range(2):
                acc.acc_spmm_execute(plan, B, w.N, C, stream)
            torch.cuda.synchronize()
            ts = [sum(acc.acc_spmm_execute_timed(plan, B, w.N, C, stream)) for _ in range(args.steps)]
        finally:
            acc.acc_spmm_destroy(plan)
        ms = float(np.mean(ts))
        return ms, 2.0 * w.nnz * w.N / (ms * 1e-3) / 1e9, st

    # --- format (Section 4.3.2), paper geometry 8x8, with and without reordering
    for ro in (OFF, ON):
        plan = plan_with(window_height=8, tile_width=8, reorder=ro)
        st = acc.acc_spmm_plan_stats(plan)
        acc.acc_spmm_destroy(plan)
        W, T = st["num_windows"], st["num_tiles"]
        csr = 4 * (w.M + 1) + 4 * w.nnz
        int8_tiles = 4 * (W + 1) + 4 * (T + 1) + 4 * 8 * T + w.nnz          # one int8 local id per entry
        bitmap_tiles = st["index_bytes"]
        print(json.dumps({"report": "format-8x8", "workload": w.name, "reordered": bool(ro), "tiles": T,
                          "mean_nnz_per_tile": st["mean_nnz_per_tile"], "index_bytes_csr": csr,
                          "index_bytes_int8_local_id_tiles": int8_tiles, "index_bytes_bitmap_tiles": bitmap_tiles,
                          "bitmap_vs_csr": bitmap_tiles / csr, "bitmap_vs_int8": bitmap_tiles / int8_tiles}), flush=True)

    # --- ablation (Section 4.3.5 order: reordering, cache policy, pipeline, load balancing; then the
    #     column order, which the paper leaves as future work)
    steps = [
        ("base: tiles only", dict(reorder=OFF, load_balance=OFF, column_order=OFF, no_prefetch=1, streaming_stores=1)),
        ("+ reordering", dict(reorder=ON, load_balance=OFF, column_order=OFF, no_prefetch=1, streaming_stores=1)),
        ("+ cache policy (ordinary C stores)", dict(reorder=ON, load_balance=OFF, column_order=OFF, no_prefetch=1)),
        ("+ pipeline", dict(reorder=ON, load_balance=OFF, column_order=OFF)),
        ("+ load balancing", dict(reorder=ON, load_balance=ON, column_order=OFF)),
        ("+ column order (B gathered per call)", dict(reorder=ON, load_balance=ON, column_order=ON)),
        ("library defaults (AUTO)", dict()),
    ]
    for name, kw in steps:
        ms, gf, st = timed(**kw)
        print(json.dumps({"report": "ablation", "workload": w.name, "step": name, "ms": ms, "gflops": gf,
                          "tiles": st["num_tiles"], "items": st["num_items"], "ibd": st["ibd"],
                          "reorder_applied": st["reorder_applied"], "load_balance_applied": st["load_balance_applied"],
                          "column_order_applied": st["column_order_applied"]}),
              flush=True)
    # --- sampled dense-dense product on the same pattern (N = 64 and 128 features)
    plan = plan_with(keep_entry_map=1)
    try:
        st = acc.acc_spmm_plan_stats(plan)
        out = torch.empty(max(w.nnz, 1), dtype=torch.float32, device=dev)
        for N in (64, 128):
            X = torch.randint(-15000, 15000, (w.M, N), dtype=torch.int16, device=dev)
            Y = torch.randint(-15000, 15000, (w.K, N), dtype=torch.int16, device=dev)
            for _ in range(2):
                acc.acc_spmm_sddmm(plan, X, Y, N, out, 1, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                acc.acc_spmm_sddmm(plan, X, Y, N, out, 1, stream)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            # rows of Y gathered per window, X once, results and their entry map, the format's index arrays
            alg = st["sum_distinct_cols"] * N * 2 + w.M * N * 2 + 8 * w.nnz + 2 * w.nnz + st["index_bytes"]
            print(json.dumps({"report": "sddmm", "workload": w.name, "N": N, "ms": ms,
                              "gflops": 2.0 * w.nnz * N / (ms * 1e-3) / 1e9, "algorithmic_bytes": alg,
                              "GBps": alg / (ms * 1e-3) / 1e9, "frac_of_8TBps": alg / (ms * 1e-3) / 8e12}), flush=True)
            del X, Y
    finally:
        acc.acc_spmm_destroy(plan)
    return 0


def variants(args, torch, acc, wl) -> int:
    """One JSON line per width: whole execute in ms (median of --steps launches) for the library's own choice and for
    every forced form that the width allows."""
    w = wl.config(args.config, args.shrink, with_B=False)
    forms = [("default", {}), ("fetch per-lane", dict(value_fetch=1)), ("fetch cooperative", dict(value_fetch=2)),
             ("fetch span", dict(value_fetch=3)), ("one slab per wave", dict(slabs_per_wave=1)),
             ("two slabs per wave", dict(slabs_per_wave=2)), ("ring depth 1", dict(pipeline_depth=1)),
             ("ring depth 2", dict(pipeline_depth=2)), ("ring depth 3", dict(pipeline_depth=3)),
             ("no prefetch", dict(no_prefetch=1)), ("16x32 tiles, depth 1", dict(tile_width=32, pipeline_depth=1)),
             ("16x32 tiles, depth 2", dict(tile_width=32, pipeline_depth=2)), ("LDS staging", dict(lds_staging=1))]
    plans = {name: acc.acc_spmm_plan_ex(w.M, w.K, w.nnz, w.rowptr, w.colidx, w.vals, acc.make_options(**kw)) for name, kw in forms}
    stream = torch.cuda.current_stream().cuda_stream
    try:
        for N in (int(x) for x in args.widths.split(",")):
            B = torch.from_numpy(wl.dense(w.K, N, wl.SEED_BASE, "normal", 0.0, 1.0).view(np.int16)).cuda()
            C = torch.empty((w.M, N), dtype=torch.float32, device="cuda")
            ms = {}
            for name, plan in plans.items():
                try:
                    for _ in range(2):
                        acc.acc_spmm_execute(plan, B, N, C, stream)
                except acc.AccSpmmError:
                    continue                  # a form that does not exist at this width (LDS staging, mostly)
                torch.cuda.synchronize()
                ms[name] = round(float(np.median([sum(acc.acc_spmm_execute_timed(plan, B, N, C, stream))
                                                  for _ in range(args.steps)])), 4)
            print(json.dumps({"report": "variants", "workload": w.name, "N": N, "execute_ms": ms}), flush=True)
            del B, C
            torch.cuda.empty_cache()
    finally:
        for plan in plans.values():
            acc.acc_spmm_destroy(plan)
    return 0


if __name__ == "__main__":
    sys.exit(main())
