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

# HBM bytes per launch measured with rocprofv3 (FETCH_SIZE + WRITE_SIZE, scaled by the copy-probe factors);
# source: profiles/c3_epoch_hbm_traffic.md.  Keyed by (workload, kernel as named in the roofline object).
MEASURED_TRAFFIC_BYTES = {
    ("c3", "dual_multi_kernel<128, 2>"): 2.0 * 24195312 * 1024 + 1516525 * 1024,   # 51.1 GB (second gather included)
    ("c3", "dual_rows_kernel<128>"): 2.0 * 8965572 * 1024 + 2064917 * 1024,        # 20.5 GB
}
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
    prm = als.make_params(p.alpha, p.lam, path=als.PATH_PRIMAL if args.path == "primal" else als.PATH_AUTO)
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

    # ---- roofline of the dominant kernel (largest share of the timed region) ----------------------
    # Algorithmic work, per launch, of the kernels that can dominate:
    #   dual row kernel of class c (rows with 16c < k <= 16(c+1)):  HBM-bound,
    #       bytes = nnz_c*(4*d + 4) [gathered fp32 rows of Z + column ids]
    #             + rows_c*(4*d + 8 + 4) [r store, indptr, list entry]
    #   primal fused kernel (rows beyond the dual range):  fp32-MFMA-bound,
    #       flops = 2*nnz_p*d^2 + rows_p*(d^3/3 + 2*d^2)
    #   table transform (Z = V L^-T and X = R L^-1):  HBM-bound, bytes = rows*d*(s_in + s_out)
    #   Gramian: fp32-MFMA-bound, flops = 2*rows*d^2
    # Counts are summed over the launches of the timed region and divided by the launch count.
    nsteps = max(args.steps, 1)
    deg = {"row": p.indptr[1:] - p.indptr[:-1], "col": p.t_indptr[1:] - p.t_indptr[:-1]}
    dual_max = 0 if args.path == "primal" else {16: 16, 32: 32, 64: 64, 128: 128}[d]
    cls_rows, cls_nnz = [0] * 8, [0] * 8
    prim_rows = prim_nnz = 0
    for kdeg in deg.values():
        for c in range(8):
            msk = (kdeg > 16 * c) & (kdeg <= min(16 * (c + 1), dual_max))
            cls_rows[c] += int(msk.sum())
            cls_nnz[c] += int(kdeg[msk].sum())
        msk = (kdeg > dual_max) & (kdeg <= 512)
        prim_rows += int(msk.sum())
        prim_nnz += int(kdeg[msk].sum())
    cand = {}
    for c in range(8):
        ms, launches = stage_ms.get(f"dual_k{16 * (c + 1)}", 0.0), stage_ms.get(f"launches_k{16 * (c + 1)}", 0.0)
        if launches > 0:
            kname = {0: f"dual_rows_kernel<{d}>", 1: f"dual_multi_kernel<{d}, 2>"}.get(c, f"dual_wide_kernel<{d}, {c + 1}>")
            per_launch = nsteps * (cls_nnz[c] * (4 * d + 4) + cls_rows[c] * (4 * d + 12)) / launches
            cand[kname] = (ms, launches, "hbm", per_launch)
    if stage_ms.get("primal", 0) > 0:
        fl = nsteps * (2.0 * prim_nnz * d * d + prim_rows * (d ** 3 / 3.0 + 2.0 * d * d)) / (2 * nsteps)
        cand[f"primal_kernel<{d}>"] = (stage_ms["primal"], 2 * nsteps, "mfma", fl)
    if stage_ms.get("transform", 0) > 0:
        # per half: factor (negligible) + Z transform (rows*d*(es+4)) + X transform (rows*d*(4+es)), timed together
        by = 0.5 * (m + n) * d * (es + 4) * 2
        cand[f"transform_kernel<{d}> (both passes of a half-epoch)"] = (stage_ms["transform"], 2 * nsteps, "hbm", by)
    if stage_ms.get("gramian", 0) > 0:
        cand[f"gramian_partial_kernel<{d}>"] = (stage_ms["gramian"], 2 * nsteps, "mfma", 2.0 * 0.5 * (m + n) * d * d)
    dom = max(cand, key=lambda kk: cand[kk][0])
    dom_ms_total, dom_launches, bound, work = cand[dom]
    dom_ms = dom_ms_total / dom_launches
    if bound == "hbm":
        ach = work / (dom_ms * 1e-3) / 1e9
        roof = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": None}
    else:
        ach = work / (dom_ms * 1e-3) / 1e12
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_F32_PEAK_TFLOPS, "traffic": None}
    if not args.rows:
        roof["traffic"] = MEASURED_TRAFFIC_BYTES.get((args.workload, dom))
    roof["avg_launch_ms"] = dom_ms
    roof["launches"] = dom_launches
    roof["share_of_epoch"] = dom_ms_total / nsteps / ms_per_step
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
                   "path": args.path, "row_deg_mean": stats["row_deg_mean"], "col_deg_max": stats["col_deg_max"]},
        "epoch_ms": ms_per_step, "rows_per_sec": (m + n) / (ms_per_step * 1e-3),
        "stage_ms_per_epoch": {k: round(v / max(args.steps, 1), 4) for k, v in stage_ms.items() if v > 0},
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
