#!/usr/bin/env python3
"""Benchmark of the iALS epoch (both half-epochs, both Gramians) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3]

A step is one full epoch over a synthetic link matrix that is already resident in HBM:
Gramian of H, every row of Y solved, Gramian of the new W, every row of Y^T solved.
The headline value is observed nonzeros per second (2*nnz / epoch time).  One JSON line is
printed on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from the committed counter summary
    (profiles/hbm_traffic.json, written by profile_summary.py from rocprofv3 FETCH_SIZE / WRITE_SIZE passes
    scaled by the copy-probe factors); None when that kernel was not profiled on that workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    for entry in table.get(workload, []):
        if entry["kernel"] == kernel:
            return entry["bytes_per_launch"]
    return None


HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(p, nnz, sample_rows, gram_rows):
    """Time the fp64 oracle on a bounded, seeded sample of the same workload (rank 0 only)."""
    import numpy as np
    import torch

    import oracle
    from synth import hash_u64

    d = p.d
    halves = []
    for tag, indptr, indices, V, m in (("row", p.indptr, p.indices, p.H0, p.rows),
                                       ("col", p.t_indptr, p.t_indices, p.W0, p.cols)):
        n = V.shape[0]
        g_rows = min(gram_rows, n)
        Vs = V[:g_rows].double().cpu().numpy()
        t0 = time.perf_counter()
        Gs = oracle.gramian(Vs)
        t_gram = time.perf_counter() - t0
        G = Gs * (n / g_rows)  # stand-in of the right scale; only the timing of the solve uses it
        order = torch.argsort(hash_u64(99, 17, torch.arange(m, device=indptr.device)))[:sample_rows]
        rows = torch.sort(order).values
        starts, ends = indptr[rows], indptr[rows + 1]
        lens = (ends - starts)
        sub_ptr = torch.zeros(rows.numel() + 1, dtype=torch.int64, device=indptr.device)
        torch.cumsum(lens, 0, out=sub_ptr[1:])
        pos = torch.repeat_interleave(starts - sub_ptr[:-1], lens) + torch.arange(int(sub_ptr[-1]), device=indptr.device)
        sub_idx = indices[pos]
        uniq, inv = torch.unique(sub_idx, return_inverse=True)
        Vsub = V[uniq.long()].double().cpu().numpy()
        ip, ix = sub_ptr.cpu().numpy(), inv.to(torch.int32).cpu().numpy()
        t0 = time.perf_counter()
        oracle.solve_rows(ip, ix, None, Vsub, G, p.alpha, p.lam, None, "f32")
        t_rows = time.perf_counter() - t0
        nnz_s = int(sub_ptr[-1])
        halves.append(dict(tag=tag, t_gram=t_gram, g_rows=g_rows, n=n, t_rows=t_rows, rows=int(rows.numel()),
                           nnz=nnz_s, m=m))
    epoch_s = sum(h["t_gram"] * h["n"] / h["g_rows"] + h["t_rows"] * h["m"] / h["rows"] for h in halves)
    work_s = sum(h["t_gram"] + h["t_rows"] for h in halves)
    return {
        "value": 2.0 * nnz / epoch_s, "unit": "nnz/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": (f"fp64 C oracle, per half: Gramian timed on {halves[0]['g_rows']} table rows (single thread, "
                   f"scaled to the table) + Eq. 4 solve timed on {halves[0]['rows']} seeded uniformly sampled rows "
                   f"({halves[0]['nnz']}+{halves[1]['nnz']} nnz), scaled by rows; {work_s:.1f} s of CPU work; "
                   f"extrapolated epoch {epoch_s:.0f} s"),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--rows", type=int, default=0, help="override the node count (debugging only; invalidates the line)")
    ap.add_argument("--path", default="auto", choices=["auto", "primal"])
    ap.add_argument("--solver", default="direct", choices=["direct", "cg", "cg_free"],
                    help="direct (default, the headline line); cg: conjugate gradients on the dual / assembled systems; "
                         "cg_free: matrix-free conjugate gradients (solver variants of Sec. 4.5, reported beside the default)")
    ap.add_argument("--cg-tol", type=float, default=1e-6)
    ap.add_argument("--graph", action="store_true",
                    help="also time the epoch recorded once into a HIP graph and replayed (reported as graph_replay)")
    ap.add_argument("--topk-queries", type=int, default=4096,
                    help="after the timed epochs: exact top-20 of this many rows of W against all of H (0 = skip); "
                         "reported beside the headline figure, not part of it")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="run the library's plain copy kernel on this many MiB first (counter calibration when profiling)")
    ap.add_argument("--cpu-sample-rows", type=int, default=50000)
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")
        sys.exit(2)

    import torch

    from paper_2112_02194_amd import binding as als
    from synth import make_problem

    if not os.path.exists(als.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    kw = dict(rows=args.rows, cols=args.rows) if args.rows else {}
    p = make_problem(args.workload, device=dev, **kw)
    torch.cuda.synchronize()
    stats = p.stats()
    torch.cuda.empty_cache()  # the generator's temporaries go back to the driver: the library allocates with hipMalloc
    log(f"generated {args.workload} in {time.perf_counter() - t0:.1f} s: {stats}")
    nnz, d, m, n = p.nnz, p.d, p.rows, p.cols
    es = 4 if p.table_dtype == torch.float32 else 2

    ctx = als.Context(0)
    Y = als.Csr(m, n, p.indptr, p.indices)
    Yt = als.Csr(n, m, p.t_indptr, p.t_indices)
    W, H = p.W0.clone(), p.H0.clone()
    solver = {"direct": als.SOLVER_DIRECT, "cg": als.SOLVER_CG, "cg_free": als.SOLVER_CG_FREE}[args.solver]
    prm = als.make_params(p.alpha, p.lam, path=als.PATH_PRIMAL if args.path == "primal" else als.PATH_AUTO,
                          solver=solver, cg_tol=args.cg_tol if solver else 0.0)
    als.als_check_csr(ctx, Y)
    als.als_check_csr(ctx, Yt)

    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib * (1 << 18), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        als.als_copy_probe(ctx, src, dst)
        torch.cuda.synchronize()
        assert bool(torch.equal(src, dst))
        del src, dst
    for i in range(args.warmup):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
        torch.cuda.synchronize()
        log(f"warmup {i} done")
    als.als_set_timing(ctx, True)
    stage_ms, stage_launches = {}, {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # a second, untimed pass collects the per-kernel times (reading them waits for the events of every launch)
    for i in range(args.steps):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
        tm = als.als_get_timing(ctx)
        for k, v in tm.items():
            if k != "launches":
                stage_ms[k] = stage_ms.get(k, 0.0) + v
                stage_launches[k] = stage_launches.get(k, 0.0) + tm["launches"][k]
    torch.cuda.synchronize()
    als.als_set_timing(ctx, False)
    als.als_status_sync(ctx)
    ms_per_step = 1e3 * elapsed / max(args.steps, 1)
    loss = als.als_loss(ctx, Y, W, H, prm)
    log(f"{args.steps} epochs in {elapsed:.3f} s; kernel ms per epoch: "
        + ", ".join(f"{k}={v / max(args.steps, 1):.2f}" for k, v in stage_ms.items() if v > 0) + f"; loss {loss:.6g}")

    # ---- roofline per kernel ------------------------------------------------------------------------
    # Algorithmic work per epoch of each timed kernel (what the method itself must move or compute):
    #   dual row kernel of a class:  HBM-bound,  nnz_c*(s_z*d + 4) [gathered rows of Z (s_z = 4 bytes, 2 for bf16
    #                                           tables) + column ids] + rows_c*(4*d + 8 + 4) [r store, indptr, list entry]
    #   Z = V L^-T and X = R L^-1:   HBM-bound,  rows*d*(s_in + s_out) bytes
    #   Gramian:                     HBM-bound, rows*d*s bytes (d >= 64: products on the bf16 matrix cores); fp32 tables
    #                                with d < 64: fp32-MFMA-bound, 2*rows*d^2 flop
    #   primal fused rows:           fp32 tables: fp32-MFMA-bound, 2*nnz_p*d^2 + rows_p*(d^3/3 + 2*d^2) flop;
    #                                bf16 tables: the fp32 solves on the vector ALU, rows_p*(d^3/3 + 2*d^2) flop
    #   long-row segments:           fp32 tables: fp32-MFMA-bound, 2*nnz_l*d^2 flop; bf16 tables: HBM-bound gather
    # achieved = work of the launches timed / their summed duration (HIP events on the launch stream).
    nsteps = max(args.steps, 1)
    deg = {"row": p.indptr[1:] - p.indptr[:-1], "col": p.t_indptr[1:] - p.t_indptr[:-1]}
    dual_max = 0 if args.path == "primal" else {16: 16, 32: 32, 64: 64, 128: 128}[d]
    bounds = [("dual_k4", 0, 4), ("dual_k8", 4, 8)] + [(f"dual_k{16 * (c + 1)}", max(16 * c, 8), 16 * (c + 1)) for c in range(8)]
    bft = "true" if es == 2 else "false"  # the kernels' template arguments as rocprofv3 prints them
    zbt = "true" if (es == 2 and d >= 32) else "false"  # Z kept as bf16
    kernel_names = {"dual_k4": f"dual_small_kernel<{d},4,{zbt},false>", "dual_k8": f"dual_small_kernel<{d},8,{zbt},false>",
                    "dual_k16": f"dual_rows_kernel<{d},{zbt},false>", "dual_k32": f"dual_multi_kernel<{d},2,{zbt},false>"}
    for c in range(2, 8):
        kernel_names[f"dual_k{16 * (c + 1)}"] = f"dual_wide_kernel<{d},{c + 1},{zbt},false,false>"
    if args.solver == "cg" and d >= 64:  # every class runs the one-row-per-wavefront kernel with the CG solver
        for name, _, hi in bounds:
            kernel_names[name] = f"dual_wide_kernel<{d},{max(3, hi // 16)},{zbt},true,true>"
    if args.solver == "cg_free":
        for name, _, _ in bounds:
            kernel_names[name] = f"cg_free_kernel<{d},{bft}>"
    kernel_names.update({"gramian": (f"gramian_bf16_kernel<{d}>" if es == 2 else f"gramian_split_kernel<{d}>") if d >= 64
                         else f"gramian_partial_kernel<{d},{bft}>",
                         "transform_z": f"transform16_kernel<{d},true,true>" if zbt == "true"      # Z = V L^-T
                         else f"transform_kernel<{d},{bft},false,true>",
                         "transform_x": f"transform16_kernel<{d},false,false>" if zbt == "true"    # X = R L^-1
                         else (f"transform_split_kernel<{d},false>" if (es == 4 and d >= 64)
                               else f"transform_kernel<{d},false,{bft},false>"),
                         "primal": f"primal_kernel<{d},{bft},0,false>",               # one workgroup per row
                         "segment": f"primal_kernel<{d},{bft},1,false>"})             # segments of long rows
    zs = 2 if (es == 2 and d >= 32) else 4  # bytes per element of the transformed table Z the dual kernels gather
    if args.solver == "cg_free":
        zs = es  # the matrix-free solver gathers the fixed table itself (at least once)
    work = {}
    long_nnz = prim_rows = prim_nnz = 0
    for kdeg in deg.values():
        for name, lo, hi in bounds:
            msk = (kdeg > lo) & (kdeg <= min(hi, dual_max))
            r_c, n_c = int(msk.sum()), int(kdeg[msk].sum())
            w = work.setdefault(name, ["hbm", 0.0])
            w[1] += n_c * (zs * d + 4) + r_c * (4 * d + 12)
        # the library's long-row threshold: 512, raised until the segments of all longer rows fit its workspace
        beyond = int(kdeg[kdeg > 512].sum())
        split = max(512, -(-beyond // 16384))
        msk = (kdeg > dual_max) & (kdeg <= split)
        prim_rows += int(msk.sum())
        prim_nnz += int(kdeg[msk].sum())
        long_nnz += int(kdeg[kdeg > split].sum())
    if es == 4:  # fp32 tables: the statistics run on the fp32 matrix cores
        work["primal"] = ["mfma", 2.0 * prim_nnz * d * d + prim_rows * (d ** 3 / 3.0 + 2.0 * d * d)]
        work["segment"] = ["mfma", 2.0 * long_nnz * d * d]
        # d >= 64: three-way split products on the bf16 matrix cores leave the table read as the bound
        work["gramian"] = ["hbm", float(m + n) * d * es] if d >= 64 else ["mfma", 2.0 * (m + n) * d * d]
    else:       # bf16 tables: statistics on the bf16 matrix cores leave the gather (HBM) and the fp32 solve (vector ALU)
        work["primal"] = ["alu", prim_rows * (d ** 3 / 3.0 + 2.0 * d * d)]
        work["segment"] = ["hbm", float(long_nnz) * (d * es + 4)]
        work["gramian"] = ["hbm", float(m + n) * d * es]
    work["transform_z"] = ["hbm", float(m + n) * d * (es + zs)]
    work["transform_x"] = ["hbm", float(m + n) * d * (4 + es)]
    stages = {}
    for name, (bound, per_epoch) in work.items():
        ms = stage_ms.get(name, 0.0) / nsteps
        if ms <= 0 or per_epoch <= 0:
            continue
        if bound == "hbm":
            ach, peak, unit = per_epoch / (ms * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        else:  # "mfma": fp32 matrix cores; "alu": fp32 vector units - the same published 157.3 TFLOP/s
            ach, peak, unit = per_epoch / (ms * 1e-3) / 1e12, MFMA_F32_PEAK_TFLOPS, "TFLOP/s"
        launches = stage_launches.get(name, 0.0) / nsteps
        stages[name] = {"kernel": kernel_names.get(name, name), "ms_per_epoch": round(ms, 4), "launches_per_epoch": launches,
                        "bound": bound, "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
                        "algorithmic_per_epoch": per_epoch}
    dom = max(stages, key=lambda kk: stages[kk]["ms_per_epoch"])
    sd = stages[dom]
    per_launch = sd["algorithmic_per_epoch"] / max(sd["launches_per_epoch"], 1.0)
    roof = {"kernel": sd["kernel"], "bound": sd["bound"], "achieved": sd["achieved"], "peak": sd["peak"], "unit": sd["unit"],
            "frac": sd["frac"], "traffic": measured_traffic(f"{args.workload}@{args.rows}" if args.rows else args.workload, sd["kernel"]),
            "avg_launch_ms": sd["ms_per_epoch"] / max(sd["launches_per_epoch"], 1.0), "launches": sd["launches_per_epoch"] * nsteps,
            "algorithmic_per_launch": per_launch,
            "share_of_epoch": sd["ms_per_epoch"] / ms_per_step}
    # whole-epoch figure against the HBM floor of the method itself (gather + ids + both tables once)
    epoch_bytes = 2 * nnz * (d * es + 4) + 2 * (m + n) * d * es + 8 * (m + n + 2)
    roof["epoch_algorithmic_GBps"] = epoch_bytes / (ms_per_step * 1e-3) / 1e9

    out = {
        "metric": "observed_nnz_per_sec", "value": 2.0 * nnz / (ms_per_step * 1e-3), "unit": "nnz/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if es == 4 else "bf16-stored/f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {m}x{n} link matrix, nnz={nnz}, d={d}, "
                               f"alpha={p.alpha}, lambda={p.lam}, 1 epoch = 2 half-epochs + 2 Gramians",
                   "path": args.path, "solver": args.solver, "row_deg_mean": stats["row_deg_mean"], "col_deg_max": stats["col_deg_max"]},
        "epoch_ms": ms_per_step, "rows_per_sec": (m + n) / (ms_per_step * 1e-3),
        "loss_after": loss,
        "roofline": roof,
        "kernels": stages,
    }
    if args.graph:
        # the epoch enqueues kernels only, so it can be recorded once and replayed: what is left of the launch
        # overhead matters for the small workloads
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            als.als_epoch(ctx, Y, Yt, W, H, prm)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        out["graph_replay"] = {"ms_per_step": 1e3 * (time.perf_counter() - t0) / max(args.steps, 1), "steps": args.steps}
        log("graph replay:", out["graph_replay"])
        als.als_status_sync(ctx)
    if args.topk_queries > 0:
        # retrieval (Sec. 4.6 / Sec. 5's evaluation): exact top-20 by inner product; 2*nq*n*d flop on the fp32 matrix cores
        nq, kk = min(args.topk_queries, m), 20
        Q = W[:nq].contiguous()
        als.als_topk(ctx, Q, H, kk)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        reps = 2
        for _ in range(reps):
            ids, _ = als.als_topk(ctx, Q, H, kk)
        e1.record()
        torch.cuda.synchronize()
        tk_ms = e0.elapsed_time(e1) / reps
        tf = 2.0 * nq * n * d / (tk_ms * 1e-3) / 1e12
        out["topk"] = {"queries": nq, "items": n, "k": kk, "ms": round(tk_ms, 3), "queries_per_sec": nq / (tk_ms * 1e-3),
                       "bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(tf / MFMA_F32_PEAK_TFLOPS, 4),
                       "item_table_GBps": round(math.ceil(nq / 64) * n * d * es / (tk_ms * 1e-3) / 1e9, 1)}
        log("top-k:", out["topk"])
    if args.rows:
        out["config"]["note"] = "node count overridden: not the named workload"
    if not args.no_cpu_baseline:
        p.W0, p.H0 = p.W0, p.H0
        out["cpu_baseline"] = cpu_baseline(p, nnz, args.cpu_sample_rows, 200000)
        log("cpu baseline:", out["cpu_baseline"])
    print(json.dumps(out), flush=True)
    ctx.close()


if __name__ == "__main__":
    main()
