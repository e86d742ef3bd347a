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
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

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
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--rows", type=int, default=0, help="override the node count (debugging only; invalidates the line)")
    ap.add_argument("--path", default="auto", choices=["auto", "primal"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    log(f"generated {args.workload} in {time.perf_counter() - t0:.1f} s: {stats}")
    nnz, d, m, n = p.nnz, p.d, p.rows, p.cols
    es = 4 if p.table_dtype == torch.float32 else 2

    ctx = als.Context(0)
    Y = als.Csr(m, n, p.indptr, p.indices)
    Yt = als.Csr(n, m, p.t_indptr, p.t_indices)
    W, H = p.W0.clone(), p.H0.clone()
    prm = als.make_params(p.alpha, p.lam, path=als.PATH_PRIMAL if args.path == "primal" else als.PATH_AUTO)
    als.als_check_csr(ctx, Y)
    als.als_check_csr(ctx, Yt)

    for i in range(args.warmup):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
        torch.cuda.synchronize()
        log(f"warmup {i} done")
    als.als_set_timing(ctx, True)
    stage_ms = {}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
        for k, v in als.als_get_timing(ctx).items():
            stage_ms[k] = stage_ms.get(k, 0.0) + v
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    als.als_set_timing(ctx, False)
    als.als_status_sync(ctx)
    ms_per_step = 1e3 * elapsed / max(args.steps, 1)
    loss = als.als_loss(ctx, Y, W, H, prm)
    log(f"{args.steps} epochs in {elapsed:.3f} s; stage ms (sum over steps): "
        + ", ".join(f"{k}={v:.2f}" for k, v in stage_ms.items()) + f"; loss {loss:.6g}")

    # roofline of the dominant row kernel.  Per launch (= one half-epoch) the algorithm itself needs
    #   bytes = nnz*(d*s + 4) + rows*d*s + 8*(rows+1)         (gather + ids, row store, indptr)
    #   flops = 2*nnz*d^2 + rows*(d^3/3 + 2*d^2)               (normal equations + Cholesky solve)
    # both halves of a square problem have the same counts, so per-launch = per-epoch / 2.
    launches = 2 * max(args.steps, 1)
    row_kernels = {k: stage_ms.get(k, 0.0) for k in ("dual", "primal", "segment", "reduce")}
    dom = max(row_kernels, key=row_kernels.get)
    dom_ms = row_kernels[dom] / launches
    bytes_launch = nnz * (d * es + 4) + 0.5 * (m + n) * d * es + 8 * (0.5 * (m + n) + 1)
    flops_launch = 2.0 * nnz * d * d + 0.5 * (m + n) * (d ** 3 / 3.0 + 2.0 * d * d)
    if dom == "dual":
        ach = bytes_launch / (dom_ms * 1e-3) / 1e9
        roof = {"kernel": "dual_rows_kernel", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": None}
    else:
        ach = flops_launch / (dom_ms * 1e-3) / 1e12
        roof = {"kernel": "primal_kernel", "bound": "mfma", "achieved": ach, "peak": MFMA_F32_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": ach / MFMA_F32_PEAK_TFLOPS, "traffic": None}
    roof["avg_launch_ms"] = dom_ms

    out = {
        "metric": "observed_nnz_per_sec", "value": 2.0 * nnz / (ms_per_step * 1e-3), "unit": "nnz/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if es == 4 else "bf16-stored/f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {m}x{n} link matrix, nnz={nnz}, d={d}, "
                               f"alpha={p.alpha}, lambda={p.lam}, 1 epoch = 2 half-epochs + 2 Gramians",
                   "path": args.path, "row_deg_mean": stats["row_deg_mean"], "col_deg_max": stats["col_deg_max"]},
        "epoch_ms": ms_per_step, "rows_per_sec": (m + n) / (ms_per_step * 1e-3),
        "stage_ms_per_epoch": {k: v / max(args.steps, 1) for k, v in stage_ms.items()},
        "loss_after": loss,
        "roofline": roof,
    }
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
