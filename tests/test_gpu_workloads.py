"""GPU parity on the shapes of the larger configurations.

Scaled-down versions of configurations 2-5 are compared with the oracle on every row; each of them is
also run at its full size, in the launch configuration bench.py times, and checked on sampled rows (rows
are independent given the fixed table and its Gramian, so a sample is an exact check of those rows).
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import f64, host_csr, max_row_err, rel_fro, say, to_dev
from paper_2112_02194_amd import binding as als
from synth import extract_rows, hash_u64, make_problem

pytestmark = pytest.mark.gpu
TOL = {torch.float32: 1e-4, torch.bfloat16: 1e-2}


@pytest.fixture(scope="module")
def ctx(gpu_device):
    c = als.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("kind,rows,dtype", [("c2", 40000, None), ("c3", 60000, None), ("c4", 80000, None),
                                             ("c5", 40000, None), ("c2", 40000, "bf16"), ("c3", 60000, "bf16"),
                                             ("c4", 80000, "bf16")])
def test_scaled_configuration_one_epoch(ctx, gpu_device, kind, rows, dtype):
    """One full epoch (both halves, both Gramians) and the loss, every row compared; configurations 2-4 also with
    bf16-stored tables (the precision policy of the paper's Section 4.4 on their shapes)."""
    say(f"scaled {kind} rows={rows} dtype={dtype or 'as configured'}")
    p = make_problem(kind, rows=rows, cols=rows, dtype=dtype)
    Y, Yt = to_dev(p, gpu_device)
    W, H = p.W0.to(gpu_device), p.H0.to(gpu_device)
    prm = als.make_params(p.alpha, p.lam)
    als.als_epoch(ctx, Y, Yt, W, H, prm)
    als.als_status_sync(ctx)
    lg = als.als_loss(ctx, Y, W, H, prm)
    storage = "f32" if p.table_dtype == torch.float32 else "bf16"
    Yh, Yth = host_csr(p.indptr, p.indices, None), host_csr(p.t_indptr, p.t_indices, None)
    Wo, Ho = oracle.epoch(Yh, Yth, f64(p.W0), f64(p.H0), p.alpha, p.lam, storage=storage)
    lo = oracle.loss(Yh, Wo, Ho, p.alpha, p.lam)
    tol = TOL[p.table_dtype]
    say(f"  {kind}: errW {rel_fro(f64(W), Wo):.2e} errH {rel_fro(f64(H), Ho):.2e} loss rel {abs(lg - lo) / abs(lo):.2e} "
        f"max deg rows {int((p.indptr[1:] - p.indptr[:-1]).max())} cols {int((p.t_indptr[1:] - p.t_indptr[:-1]).max())}")
    assert rel_fro(f64(W), Wo) <= tol and rel_fro(f64(H), Ho) <= tol
    assert max_row_err(f64(W), Wo) <= tol and max_row_err(f64(H), Ho) <= tol
    assert abs(lg - lo) <= tol * abs(lo)


def _sample_rows(indptr, n_uniform, n_per_stratum, n_long, seed):
    dev = indptr.device
    k = indptr[1:] - indptr[:-1]
    m = k.numel()
    order = torch.argsort(hash_u64(seed, 31, torch.arange(m, device=dev)))
    picks = [order[:n_uniform]]
    for lo, hi in ((0, 0), (1, 1), (2, 2), (16, 17), (32, 33), (48, 49), (64, 65), (128, 129)):
        cand = order[((k[order] >= lo) & (k[order] <= hi))]
        picks.append(cand[:n_per_stratum])
    long_rows = torch.nonzero(k > 512).flatten()
    if long_rows.numel():
        by_len = long_rows[torch.argsort(k[long_rows], descending=True)]
        picks.append(by_len[:4])                      # the largest hubs
        picks.append(by_len[4:][:: max(1, (by_len.numel() - 4) // max(n_long, 1))][:n_long])
    return torch.unique(torch.cat(picks))


class _HostChunks:
    """Row slices of a device table as fp64 numpy arrays, so that the oracle's chunked Gramian can walk
    a table that is too large to copy to the host in one piece (or is stored as bf16)."""

    def __init__(self, t):
        self.t, self.shape = t, tuple(t.shape)

    def __getitem__(self, sl):
        return self.t[sl].double().cpu().numpy()


FULL = {  # kind: (uniformly sampled rows per half, rows per stratum, long rows besides the four largest)
    "c2": (100000, 1500, 40),
    "c3": (100000, 1500, 40),
    "c4": (100000, 1500, 40),
    "c5": (100000, 1500, 40),
}


@pytest.mark.parametrize("kind", ["c2", "c3", "c4", "c5"])
def test_configuration_full_size_sampled(ctx, gpu_device, kind):
    """The named configuration at its full size (c5: 100M x 100M, 2.5e9 entries, bf16 tables), defaults as in
    bench.py: Gramians checked in full, solved rows on a seeded sample (uniform rows, the k = 0, 1, 2 strata, the
    strata at the row-class boundaries, the largest rows and a spread of the other long ones)."""
    import time
    t0 = time.time()
    say(f"{kind} full size: generate")
    p = make_problem(kind, device=gpu_device)
    torch.cuda.synchronize()
    say(f"{kind} full size: generated in {time.time() - t0:.1f} s: {p.stats()}")
    Y = als.Csr(p.rows, p.cols, p.indptr, p.indices)
    Yt = als.Csr(p.cols, p.rows, p.t_indptr, p.t_indices)
    als.als_check_csr(ctx, Y)
    als.als_check_csr(ctx, Yt)
    prm = als.make_params(p.alpha, p.lam)
    W, H = p.W0, p.H0  # updated in place: the column half sees the W just solved
    storage = "f32" if p.table_dtype == torch.float32 else "bf16"
    tol = TOL[p.table_dtype]
    n_uniform, n_stratum, n_long = FULL[kind]
    for tag, M, V, X in (("row half", Y, H, W), ("column half", Yt, W, H)):
        t0 = time.time()
        say(f"{kind} full size: {tag}")
        G = als.als_gramian(ctx, V)
        Gref = oracle.gramian_matmul(_HostChunks(V))
        assert np.abs(f64(G) - Gref).max() <= 1e-5 * np.abs(Gref).max()
        say(f"  {tag}: Gramian checked, {time.time() - t0:.1f} s")
        als.als_solve_rows(ctx, M, V, G, prm, X)
        als.als_status_sync(ctx)
        rows = _sample_rows(M.indptr, n_uniform, n_stratum, n_long, seed=5)
        sp, si, _, used = extract_rows(M.indptr, M.indices, None, rows)
        Vsub = V[used].double().cpu().numpy()
        ref = oracle.solve_rows(sp.cpu().numpy(), si.cpu().numpy(), None, Vsub, Gref, p.alpha, p.lam, None, storage)
        got = f64(X[rows])
        kk = (M.indptr[rows + 1] - M.indptr[rows]).cpu().numpy()
        say(f"  {tag}: {rows.numel()} rows sampled (k from {kk.min()} to {kk.max()}, {int(sp[-1])} entries): "
            f"rel err {rel_fro(got, ref):.2e}, worst row {max_row_err(got, ref):.2e}, {time.time() - t0:.1f} s")
        assert rel_fro(got, ref) <= tol
        assert max_row_err(got, ref) <= tol
        assert np.all(got[kk == 0] == 0.0)
        del Vsub, ref, got, G
    del p, Y, Yt, W, H, M, V, X
    torch.cuda.empty_cache()
