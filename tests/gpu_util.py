"""Helpers shared by the GPU parity tests."""
import sys

import numpy as np
import torch

from paper_2112_02194_amd import binding as als


def say(msg):
    """Name the case before it touches the GPU, flushed, so a fault can be traced to it."""
    print("[gpu-case]", msg, flush=True)
    sys.stdout.flush()


def to_dev(p, dev):
    Y = als.Csr(p.rows, p.cols, p.indptr.to(dev), p.indices.to(dev), None if p.values is None else p.values.to(dev))
    Yt = als.Csr(p.cols, p.rows, p.t_indptr.to(dev), p.t_indices.to(dev),
                 None if p.t_values is None else p.t_values.to(dev))
    return Y, Yt


def host_csr(indptr, indices, values):
    return indptr.cpu().numpy(), indices.cpu().numpy(), None if values is None else values.cpu().numpy()


def rel_fro(x, ref):
    x, ref = np.asarray(x, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(x - ref) / max(np.linalg.norm(ref), 1e-300))


def max_row_err(x, ref, floor=1e-3):
    """Largest per-row relative error; rows whose reference norm is below `floor` times the
    typical row norm are compared against that floor instead."""
    x, ref = np.asarray(x, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    rn = np.linalg.norm(ref, axis=1)
    scale = np.maximum(rn, floor * max(float(np.median(rn[rn > 0])) if np.any(rn > 0) else 1.0, 1e-300))
    return float((np.linalg.norm(x - ref, axis=1) / scale).max())


def f64(t: torch.Tensor):
    return t.detach().cpu().double().numpy()
