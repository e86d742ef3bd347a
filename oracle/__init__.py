"""ctypes loader for the CPU oracle (TEST INFRASTRUCTURE, not product code).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It wraps ``als_oracle.c`` (plain fp64 C, OpenMP over rows), which
follows the paper's Eq. 3, Eq. 4 and Algorithm 1 and shares nothing with the
HIP library.  All arrays are numpy, on the host.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "als_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

STORAGE = {"f64": 0, "f32": 1, "bf16": 2}


def build() -> str:
    """Compile the oracle with gcc; returns the library path."""
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        build()
    lib = ctypes.CDLL(_LIB)
    p = ctypes.c_void_p
    i64, i32, f64 = ctypes.c_int64, ctypes.c_int, ctypes.c_double
    lib.oracle_gramian.argtypes = [p, i64, i32, p]
    lib.oracle_gramian.restype = i32
    lib.oracle_solve_rows.argtypes = [p, p, p, p, i32, p, f64, f64, p, i64, i32, p]
    lib.oracle_solve_rows.restype = i32
    lib.oracle_epoch.argtypes = [p, p, p, p, p, p, i64, i64, i32, f64, f64, i32, p, p]
    lib.oracle_epoch.restype = i32
    for name in ("oracle_loss", "oracle_loss_literal"):
        fn = getattr(lib, name)
        fn.argtypes = [p, p, p, i64, i64, p, p, i32, f64, f64]
        fn.restype = f64
    lib.oracle_round_storage.argtypes = [p, i64, i32]
    lib.oracle_round_storage.restype = None
    lib.oracle_num_threads.argtypes = []
    lib.oracle_num_threads.restype = i32
    _lib = lib
    return lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _csr(indptr, indices, values):
    ip = np.ascontiguousarray(np.asarray(indptr, dtype=np.int64))
    ix = np.ascontiguousarray(np.asarray(indices, dtype=np.int32))
    vv = None if values is None else np.ascontiguousarray(np.asarray(values, dtype=np.float32))
    assert ip[0] == 0 and ip[-1] == ix.size and (vv is None or vv.size == ix.size)
    return ip, ix, vv


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def round_storage(x, storage: str):
    out = _f64(x).copy()
    _load().oracle_round_storage(_ptr(out), out.size, STORAGE[storage])
    return out


def gramian(V):
    V = _f64(V)
    n, d = V.shape
    G = np.empty((d, d), dtype=np.float64)
    _load().oracle_gramian(_ptr(V), n, d, _ptr(G))
    return G


def gramian_matmul(V, chunk: int = 1 << 20):
    """G = V^T V with the library matmul in fp64, chunked over rows: the same definition as
    ``gramian`` with a library primitive as the step, for tables too large for the plain loop."""
    d = V.shape[1]
    G = np.zeros((d, d), dtype=np.float64)
    for r0 in range(0, V.shape[0], chunk):
        blk = np.asarray(V[r0:r0 + chunk], dtype=np.float64)
        G += blk.T @ blk
    return G


def solve_rows(indptr, indices, values, V, G, alpha, lam, row_ids=None, storage="f64"):
    """Eq. 4 for the listed rows (all rows if ``row_ids`` is None) -> [nrows x d] fp64."""
    ip, ix, vv = _csr(indptr, indices, values)
    V, G = _f64(V), _f64(G)
    d = V.shape[1]
    if ix.size:
        assert 0 <= int(ix.min()) and int(ix.max()) < V.shape[0]
    rid = None if row_ids is None else np.ascontiguousarray(np.asarray(row_ids, dtype=np.int64))
    nrows = ip.size - 1 if rid is None else rid.size
    X = np.empty((nrows, d), dtype=np.float64)
    rc = _load().oracle_solve_rows(_ptr(ip), _ptr(ix), _ptr(vv), _ptr(V), d, _ptr(G), float(alpha),
                                   float(lam), _ptr(rid), nrows, STORAGE[storage], _ptr(X))
    if rc != 0:
        raise FloatingPointError(f"oracle_solve_rows failed with status {rc}")
    return X


def half_epoch(indptr, indices, values, V, alpha, lam, storage="f64"):
    return solve_rows(indptr, indices, values, V, gramian(V), alpha, lam, None, storage)


def epoch(Y, Yt, W, H, alpha, lam, storage="f64"):
    """One epoch; ``Y`` and ``Yt`` are (indptr, indices, values) triples.  Returns new (W, H)."""
    ip, ix, vv = _csr(*Y)
    tp, tx, tv = _csr(*Yt)
    W, H = _f64(W).copy(), _f64(H).copy()
    m, d = W.shape
    n = H.shape[0]
    rc = _load().oracle_epoch(_ptr(ip), _ptr(ix), _ptr(vv), _ptr(tp), _ptr(tx), _ptr(tv), m, n, d,
                              float(alpha), float(lam), STORAGE[storage], _ptr(W), _ptr(H))
    if rc != 0:
        raise FloatingPointError(f"oracle_epoch failed with status {rc}")
    return W, H


def loss(Y, W, H, alpha, lam, literal=False):
    """Eq. 3; ``literal`` evaluates the all-pairs term as the printed double sum."""
    ip, ix, vv = _csr(*Y)
    W, H = _f64(W), _f64(H)
    m, d = W.shape
    n = H.shape[0]
    fn = _load().oracle_loss_literal if literal else _load().oracle_loss
    return float(fn(_ptr(ip), _ptr(ix), _ptr(vv), m, n, _ptr(W), _ptr(H), d, float(alpha), float(lam)))


def topk(Q, H, k, exclude=None):
    """Exact top-k by inner product, the plain definition: all scores Q H^T in fp64, per query the k largest,
    equal scores by ascending id; `exclude` = (indptr, indices) of ids never returned per query.
    Returns (ids [nq, k] with -1 where fewer than k rows are admissible, scores [nq, k] with -inf there)."""
    Q, H = _f64(Q), _f64(H)
    S = Q @ H.T
    if exclude is not None:
        ip, ix = np.asarray(exclude[0]), np.asarray(exclude[1])
        for q in range(Q.shape[0]):
            S[q, ix[ip[q]:ip[q + 1]]] = -np.inf
    order = np.argsort(-S, axis=1, kind="stable")[:, :k]  # stable: equal scores stay in id order
    sc = np.take_along_axis(S, order, axis=1)
    ids = np.where(np.isfinite(sc), order, -1).astype(np.int64)
    if ids.shape[1] < k:
        pad = k - ids.shape[1]
        ids = np.pad(ids, ((0, 0), (0, pad)), constant_values=-1)
        sc = np.pad(sc, ((0, 0), (0, pad)), constant_values=-np.inf)
    return ids, sc


def recall_at_k(ids, held_indptr, held_indices):
    """Recall@K per query: |top-K ids that are held-out links| / min(K, number of held-out links); queries
    without a held-out link are left out (NaN)."""
    ids = np.asarray(ids)
    ip, ix = np.asarray(held_indptr), np.asarray(held_indices)
    out = np.full(ids.shape[0], np.nan)
    for q in range(ids.shape[0]):
        want = set(ix[ip[q]:ip[q + 1]].tolist())
        if want:
            out[q] = len(want.intersection(ids[q].tolist())) / min(ids.shape[1], len(want))
    return out
