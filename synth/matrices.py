"""Counter-based generators for the synthetic link matrices and embedding tables.

Every random number is a pure function ``hash(seed, stream, a, b)`` of integer
counters (a splitmix64-style mixer written with wrapping int64 torch ops), so a
matrix is reproducible on any torch device and needs no generator state.

The matrices stand in for the WebGraph link matrices of the paper's Section 5
(square, heavy-tailed out-degrees, host locality), at the shapes the benchmark
configurations name; they hold no item of that dataset.

Recipes (degrees -> column ids), one per configuration key:

``c1``  2000 x 1500; degrees: Zipf(1.1) truncated to 1..200; columns: Zipf(1.1)
        over ranks, rank -> id through a seeded permutation.
``c2``  1M x 1M; degrees: round(Pareto, pdf ~ k^-2.1 on [k_min, 5000]) with k_min
        chosen so the mean is 30; columns uniform.
``c3``  10M x 10M; degrees: shifted geometric, mean 20, clipped to [1, 2000];
        nodes grouped into 100k contiguous "hosts" with lognormal sizes; an edge
        lands inside the source's host with probability 0.8, else on a
        Zipf(1.0)-popular node.
``c4``  50M x 50M; degrees geometric, mean 6, max 1000; columns uniform.
``c5``  100M x 100M; degrees round(Pareto, pdf ~ k^-2.5 on [k_min, 1e5]), mean 25;
        columns uniform.

Zipf(s) over ranks 1..N is drawn as floor of the continuous density x^-s on
[1, N+1), which has the same tail and needs no table.

Column ids inside a row are distinct.  ``c2`` .. ``c5`` redraw a colliding slot
(attempt t of slot (row, j) is again a pure hash of (seed, t, row, j)) until the
row holds as many distinct ids as its drawn degree, so the realised degrees are
the drawn ones; ``c1`` drops duplicate pairs instead, which is what brings its
clipped-Zipf mean of 27.8 down to the "about 20" its statement names.

Matrices are built in blocks of rows (no single sort sees more than ``BLOCK``
keys) and transposed by column ranges, so 100M x 100M with 2.5e9 entries fits
the 2^31-element limits of the sorting primitives.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import torch

_MASK63 = (1 << 63) - 1


def _to_i64(x: int) -> int:
    """Reinterpret an unsigned 64-bit constant as the signed value torch wants."""
    x &= (1 << 64) - 1
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _to_i64(0x9E3779B97F4A7C15)
_C2 = _to_i64(0xBF58476D1CE4E5B9)
_C3 = _to_i64(0x94D049BB133111EB)
_C4 = _to_i64(0xD6E8FEB86659FD93)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 30)) * _C2
    z = (z ^ _lsr(z, 27)) * _C3
    return z ^ _lsr(z, 31)


def hash_u64(seed: int, stream: int, a: torch.Tensor, b: torch.Tensor | int = 0) -> torch.Tensor:
    """64 hashed bits (as int64) for every element of counters ``a`` (and ``b``)."""
    a = a.to(torch.int64)
    k = _to_i64((seed * 0x9E3779B97F4A7C15) ^ (stream * 0xD6E8FEB86659FD93))
    z = _mix(a * _C1 + k)
    if isinstance(b, torch.Tensor):
        b = b.to(torch.int64)
        z = _mix(z ^ (b * _C4 + _C1))
    else:
        z = _mix(z ^ _to_i64(b * 0xD6E8FEB86659FD93 + 0x9E3779B97F4A7C15))
    return z


def uniform01(h: torch.Tensor) -> torch.Tensor:
    """Hashed bits -> float64 uniform in (0, 1) (never exactly 0 or 1)."""
    return (_lsr(h, 11).to(torch.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal(seed: int, stream: int, a: torch.Tensor, b) -> torch.Tensor:
    u1 = uniform01(hash_u64(seed, stream, a, b))
    u2 = uniform01(hash_u64(seed, stream + 1, a, b))
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)


def init_table(rows: int, d: int, seed: int, stream: int, device="cpu",
               dtype=torch.float32, chunk: int = 1 << 22) -> torch.Tensor:
    """Embedding table with entries N(0, sigma), sigma = 0.1 / sqrt(d)."""
    out = torch.empty((rows, d), dtype=dtype, device=device)
    sigma = 0.1 / math.sqrt(d)
    col = torch.arange(d, device=device, dtype=torch.int64)[None, :]
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        r = torch.arange(r0, r1, device=device, dtype=torch.int64)[:, None]
        out[r0:r1] = (sigma * _normal(seed, stream, r * d + col, 0)).to(dtype)
    return out


# --------------------------------------------------------------------------- degrees

def _pareto_inv(u: torch.Tensor, a: float, lo: float, hi: float) -> torch.Tensor:
    """Inverse CDF of the density x^-a on [lo, hi] (a != 1)."""
    e = 1.0 - a
    lo_e, hi_e = lo ** e, hi ** e
    return (lo_e - u * (lo_e - hi_e)) ** (1.0 / e)


def _pareto_mean(a: float, lo: float, hi: float) -> float:
    e1, e2 = 1.0 - a, 2.0 - a
    return ((hi ** e2 - lo ** e2) / e2) / ((hi ** e1 - lo ** e1) / e1)


def _pareto_kmin(a: float, hi: float, mean: float) -> float:
    lo, up = 0.5, mean
    for _ in range(200):
        mid = 0.5 * (lo + up)
        if _pareto_mean(a, mid, hi) < mean:
            lo = mid
        else:
            up = mid
    return 0.5 * (lo + up)


def _zipf_rank(u: torch.Tensor, s: float, n: int) -> torch.Tensor:
    """Rank in 1..n with P(r) ~ r^-s (floor of the continuous law on [1, n+1))."""
    if abs(s - 1.0) < 1e-12:
        x = torch.exp(u * math.log(n + 1.0))
    else:
        x = _pareto_inv(u, s, 1.0, n + 1.0)
    return torch.clamp(x.floor().to(torch.int64), 1, n)


def _geometric(u: torch.Tensor, mean: float, kmax: int) -> torch.Tensor:
    """Geometric on {1, 2, ...} with the given mean, clipped to kmax."""
    p = 1.0 / mean
    k = 1 + torch.floor(torch.log(u) / math.log(1.0 - p)).to(torch.int64)
    return torch.clamp(k, 1, kmax)


# --------------------------------------------------------------------------- CSR helpers

BLOCK = 1 << 27  # most keys handed to one sort


def csr_from_edges(rows: int, cols: int, r: torch.Tensor, c: torch.Tensor,
                   v: Optional[torch.Tensor] = None):
    """Sort edges by (row, col), drop duplicate pairs, return (indptr, indices, values).
    One sort over all edges: for edge lists below 2^31 entries."""
    if r.numel() >= 2 ** 31:
        raise ValueError("csr_from_edges sorts the edge list in one piece: at most 2^31-1 entries")
    key = r.to(torch.int64) * cols + c.to(torch.int64)
    if v is None:
        key = torch.unique(key)  # sorted, duplicates removed
        vals = None
    else:
        key, order = torch.sort(key, stable=True)
        keep = torch.ones_like(key, dtype=torch.bool)
        keep[1:] = key[1:] != key[:-1]
        key = key[keep]
        vals = v[order][keep].contiguous()
    rr = torch.div(key, cols, rounding_mode="floor")
    cc = (key - rr * cols).to(torch.int32)
    counts = torch.bincount(rr, minlength=rows)
    indptr = torch.zeros(rows + 1, dtype=torch.int64, device=key.device)
    torch.cumsum(counts, 0, out=indptr[1:])
    return indptr, cc.contiguous(), vals


def _expand_rows(indptr: torch.Tensor) -> torch.Tensor:
    rows = indptr.numel() - 1
    deg = indptr[1:] - indptr[:-1]
    return torch.repeat_interleave(torch.arange(rows, device=indptr.device, dtype=torch.int64), deg)


def _ranges(ptr: torch.Tensor, block: int):
    """Cut [0, n) into consecutive ranges [a, b) with ptr[b] - ptr[a] <= block (at least one item each)."""
    n = ptr.numel() - 1
    out, a = [], 0
    while a < n:
        b = int(torch.searchsorted(ptr, ptr[a] + block, right=True)) - 1
        b = min(max(b, a + 1), n)
        out.append((a, b))
        a = b
    return out


def transpose_csr(rows: int, cols: int, indptr, indices, values=None, block: int = BLOCK):
    """CSR of the transposed matrix (true transpose, columns sorted inside each row).

    Counting pass over the column ids, then one sort per range of columns that holds at most
    ``block`` entries; the entries of a range are picked out of the matrix chunk by chunk."""
    dev = indices.device
    nnz = indices.numel()
    counts = torch.zeros(cols, dtype=torch.int64, device=dev)
    for p0 in range(0, nnz, block):
        counts += torch.bincount(indices[p0:p0 + block], minlength=cols)
    t_indptr = torch.zeros(cols + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=t_indptr[1:])
    del counts
    t_indices = torch.empty(nnz, dtype=torch.int32, device=dev)
    t_values = None if values is None else torch.empty(nnz, dtype=values.dtype, device=dev)
    for c0, c1 in _ranges(t_indptr, block):
        keys, vals = [], []
        for p0 in range(0, nnz, block):
            idx = indices[p0:p0 + block]
            sel = torch.nonzero((idx >= c0) & (idx < c1)).flatten()
            if sel.numel() == 0:
                continue
            cc = idx[sel].to(torch.int64) - c0
            sel += p0
            rr = torch.searchsorted(indptr, sel, right=True) - 1  # the row that holds entry `sel`
            keys.append(cc * rows + rr)
            if values is not None:
                vals.append(values[sel])
        o0, o1 = int(t_indptr[c0]), int(t_indptr[c1])
        if o1 == o0:
            continue
        key = torch.cat(keys)
        del keys
        if values is None:
            key = torch.sort(key).values
        else:
            key, order = torch.sort(key)
            t_values[o0:o1] = torch.cat(vals)[order]
        t_indices[o0:o1] = (key - torch.div(key, rows, rounding_mode="floor") * rows).to(torch.int32)
    return t_indptr, t_indices, t_values


# --------------------------------------------------------------------------- problems

@dataclass
class SparseProblem:
    name: str
    rows: int
    cols: int
    d: int
    alpha: float
    lam: float
    epochs: int
    table_dtype: torch.dtype
    indptr: torch.Tensor
    indices: torch.Tensor
    values: Optional[torch.Tensor]
    t_indptr: torch.Tensor
    t_indices: torch.Tensor
    t_values: Optional[torch.Tensor]
    W0: torch.Tensor
    H0: torch.Tensor

    @property
    def nnz(self) -> int:
        return int(self.indices.numel())

    def stats(self) -> dict:
        deg = self.indptr[1:] - self.indptr[:-1]
        tdeg = self.t_indptr[1:] - self.t_indptr[:-1]
        return {
            "rows": self.rows, "cols": self.cols, "nnz": self.nnz, "d": self.d,
            "row_deg_mean": float(deg.double().mean()), "row_deg_max": int(deg.max()),
            "col_deg_mean": float(tdeg.double().mean()), "col_deg_max": int(tdeg.max()),
            "empty_rows": int((deg == 0).sum()), "empty_cols": int((tdeg == 0).sum()),
        }


CONFIGS = {
    "c1": dict(rows=2000, cols=1500, d=16, alpha=0.1, lam=1e-2, epochs=4, seed=20211201, dtype="f32"),
    "c2": dict(rows=1_000_000, cols=1_000_000, d=64, alpha=0.1, lam=1e-2, epochs=1, seed=20211202, dtype="f32"),
    "c3": dict(rows=10_000_000, cols=10_000_000, d=128, alpha=0.1, lam=1e-2, epochs=1, seed=20211203, dtype="f32"),
    "c4": dict(rows=50_000_000, cols=50_000_000, d=128, alpha=0.05, lam=1e-2, epochs=1, seed=20211204, dtype="f32"),
    "c5": dict(rows=100_000_000, cols=100_000_000, d=128, alpha=0.1, lam=1e-2, epochs=1, seed=20211205, dtype="bf16"),
}


def _degrees(kind: str, rows: int, seed: int, device) -> torch.Tensor:
    r = torch.arange(rows, device=device, dtype=torch.int64)
    u = uniform01(hash_u64(seed, 1, r))
    if kind == "c1":
        return _zipf_rank(u, 1.1, 200)
    if kind == "c2":
        kmin = _pareto_kmin(2.1, 5000.0, 30.0)
        return torch.clamp(torch.round(_pareto_inv(u, 2.1, kmin, 5000.0)).to(torch.int64), 1, 5000)
    if kind == "c3":
        return _geometric(u, 20.0, 2000)
    if kind == "c4":
        return _geometric(u, 6.0, 1000)
    if kind == "c5":
        kmin = _pareto_kmin(2.5, 1e5, 25.0)
        return torch.clamp(torch.round(_pareto_inv(u, 2.5, kmin, 1e5)).to(torch.int64), 1, 100_000)
    raise ValueError(kind)


def _permutation(n: int, seed: int, stream: int, device) -> torch.Tensor:
    h = hash_u64(seed, stream, torch.arange(n, device=device, dtype=torch.int64))
    return torch.argsort(h, stable=True)


class _ColumnSampler:
    """Column id of slot (row, j), attempt t: a pure function of (seed, t, row, j).  The tables a recipe
    needs (host boundaries, the rank -> id permutation) are built once."""

    STRIDE = 16  # hash streams of attempt t: 2 + 16 t and 5 + 16 t (attempt 0: the recipe's own streams 2 and 5)

    def __init__(self, kind: str, rows: int, cols: int, seed: int, device):
        self.kind, self.rows, self.cols, self.seed = kind, rows, cols, seed
        if kind in ("c1", "c3"):
            self.perm = _permutation(cols, seed, 7, device)
        if kind == "c3":
            nhosts = max(1, cols // 100)
            hid = torch.arange(nhosts, device=device, dtype=torch.int64)
            w = torch.exp(_normal(seed, 3, hid, 0))  # lognormal(0, 1)
            size = torch.clamp(torch.floor(w / w.sum() * cols).to(torch.int64), min=1)
            # give the rounding remainder to the largest host so sizes sum to cols
            size[torch.argmax(size)] += cols - int(size.sum())
            assert int(size.min()) >= 1
            self.size = size
            self.start = torch.zeros(nhosts + 1, dtype=torch.int64, device=device)
            torch.cumsum(size, 0, out=self.start[1:])

    def draw(self, r: torch.Tensor, j: torch.Tensor, attempt: int = 0) -> torch.Tensor:
        kind, cols, seed = self.kind, self.cols, self.seed
        u = uniform01(hash_u64(seed, 2 + self.STRIDE * attempt, r, j))
        if attempt >= 16 or kind in ("c2", "c4", "c5"):  # late attempts of every recipe: uniform over all columns
            return torch.clamp((u * cols).to(torch.int64), 0, cols - 1)
        if kind == "c1":
            return self.perm[_zipf_rank(u, 1.1, cols) - 1]
        if kind == "c3":
            host = torch.searchsorted(self.start, r, right=True) - 1
            hs, h0 = self.size[host], self.start[host]
            u2 = uniform01(hash_u64(seed, 5 + self.STRIDE * attempt, r, j))
            local = h0 + torch.clamp((u2 * (hs - 1).double()).to(torch.int64), max=torch.clamp(hs - 2, min=0))
            local = local + (local >= r).to(torch.int64)  # skip self
            popular = self.perm[_zipf_rank(u2, 1.0, cols) - 1]
            inside = (u < 0.8) & (hs > 1)
            if attempt >= 6:  # a host smaller than the row's local share can never supply distinct ids
                return popular
            return torch.where(inside, local, popular)
        raise ValueError(kind)


RESAMPLE = {"c1": False, "c2": True, "c3": True, "c4": True, "c5": True}
MAX_ATTEMPTS = 64


def _member(sorted_keys: torch.Tensor, q: torch.Tensor) -> torch.Tensor:
    if sorted_keys.numel() == 0:
        return torch.zeros_like(q, dtype=torch.bool)
    pos = torch.clamp(torch.searchsorted(sorted_keys, q), max=sorted_keys.numel() - 1)
    return sorted_keys[pos] == q


def _block_keys(sampler: _ColumnSampler, r: torch.Tensor, j: torch.Tensor, resample: bool) -> torch.Tensor:
    """Sorted distinct keys row * cols + col of one block of slots."""
    cols = sampler.cols
    key, order = torch.sort(r * cols + sampler.draw(r, j, 0), stable=True)  # of equal keys the lowest slot stays
    dup = torch.zeros_like(key, dtype=torch.bool)
    dup[1:] = key[1:] == key[:-1]
    uniq = key[~dup]
    if not resample or not bool(dup.any()):
        return uniq
    pend = order[dup]  # slots whose id is already taken in their row
    del key, order, dup
    accepted = torch.empty(0, dtype=torch.int64, device=r.device)
    for attempt in range(1, MAX_ATTEMPTS):
        if pend.numel() == 0:
            break
        rp = r[pend]
        kn = rp * cols + sampler.draw(rp, j[pend], attempt)
        ks, o2 = torch.sort(kn, stable=True)
        again = torch.zeros_like(kn, dtype=torch.bool)
        again[o2[1:]] = ks[1:] == ks[:-1]  # the same id drawn twice in this round: the later slot waits
        bad = again | _member(uniq, kn) | _member(accepted, kn)
        accepted = torch.sort(torch.cat([accepted, kn[~bad]])).values
        pend = pend[bad]
    return torch.sort(torch.cat([uniq, accepted])).values  # slots still pending after the last attempt are dropped


def build_csr(kind: str, rows: int, cols: int, seed: int, deg: torch.Tensor, block: int = BLOCK):
    """CSR of the recipe's matrix from the drawn row degrees, built in blocks of rows."""
    dev = deg.device
    sampler = _ColumnSampler(kind, rows, cols, seed, dev)
    ptr0 = torch.zeros(rows + 1, dtype=torch.int64, device=dev)
    torch.cumsum(deg, 0, out=ptr0[1:])
    indices = torch.empty(int(ptr0[-1]), dtype=torch.int32, device=dev)
    counts = torch.empty(rows, dtype=torch.int64, device=dev)
    written = 0
    for a, b in _ranges(ptr0, block):
        n = int(ptr0[b] - ptr0[a])
        r = a + torch.repeat_interleave(torch.arange(b - a, device=dev, dtype=torch.int64), deg[a:b])
        j = torch.arange(n, device=dev, dtype=torch.int64) - (ptr0[r] - ptr0[a])
        key = _block_keys(sampler, r, j, RESAMPLE[kind])
        del r, j
        rr = torch.div(key, cols, rounding_mode="floor")
        indices[written:written + key.numel()] = (key - rr * cols).to(torch.int32)
        counts[a:b] = torch.bincount(rr - a, minlength=b - a)
        written += key.numel()
        del key, rr
    indptr = torch.zeros(rows + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=indptr[1:])
    return indptr, indices[:written]


def entry_values(seed: int, indptr: torch.Tensor, indices: torch.Tensor, transposed: bool = False,
                 block: int = BLOCK) -> torch.Tensor:
    """Labels in [0.5, 1.5), a pure function of (seed, row, column) of the untransposed matrix."""
    out = torch.empty(indices.numel(), dtype=torch.float32, device=indices.device)
    for a, b in _ranges(indptr, block):
        o0, o1 = int(indptr[a]), int(indptr[b])
        deg = indptr[a + 1:b + 1] - indptr[a:b]
        r = a + torch.repeat_interleave(torch.arange(b - a, device=indices.device, dtype=torch.int64), deg)
        c = indices[o0:o1].to(torch.int64)
        if transposed:
            r, c = c, r
        out[o0:o1] = (0.5 + uniform01(hash_u64(seed, 9, r, c))).to(torch.float32)
    return out


def make_problem(kind: str, device="cpu", rows: Optional[int] = None, cols: Optional[int] = None,
                 d: Optional[int] = None, values: str = "ones", seed: Optional[int] = None,
                 dtype: Optional[str] = None, tables: bool = True) -> SparseProblem:
    """Build one synthetic problem.  ``rows``/``cols``/``d`` override the
    configuration's sizes (the recipe scales with them); ``values`` is "ones"
    (binary implicit feedback, stored as no value array) or "uniform" (labels in
    [0.5, 1.5), to exercise general y); ``tables=False`` leaves W0 and H0 out."""
    cfg = dict(CONFIGS[kind])
    rows = rows or cfg["rows"]
    cols = cols or cfg["cols"]
    d = d or cfg["d"]
    seed = cfg["seed"] if seed is None else seed
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}[dtype or cfg["dtype"]]
    deg = torch.clamp(_degrees(kind, rows, seed, device), max=cols - 1 if kind == "c3" else cols)
    indptr, indices = build_csr(kind, rows, cols, seed, deg)
    del deg
    vals = entry_values(seed, indptr, indices) if values == "uniform" else None
    t_indptr, t_indices, _ = transpose_csr(rows, cols, indptr, indices, None)
    t_vals = entry_values(seed, t_indptr, t_indices, transposed=True) if values == "uniform" else None
    W0 = init_table(rows, d, seed, 11, device=device, dtype=tdt) if tables else None
    H0 = init_table(cols, d, seed, 13, device=device, dtype=tdt) if tables else None
    return SparseProblem(kind, rows, cols, d, cfg["alpha"], cfg["lam"], cfg["epochs"], tdt,
                         indptr, indices, vals, t_indptr, t_indices, t_vals, W0, H0)


def _select_entries(indptr: torch.Tensor, indices: torch.Tensor, rows: torch.Tensor, keep: torch.Tensor):
    """CSR of the listed rows restricted to the entries flagged in `keep` (one flag per entry of the matrix)."""
    starts, lens = indptr[rows], indptr[rows + 1] - indptr[rows]
    ptr = torch.zeros(rows.numel() + 1, dtype=torch.int64, device=indptr.device)
    torch.cumsum(lens, 0, out=ptr[1:])
    pos = torch.repeat_interleave(starts - ptr[:-1], lens) + torch.arange(int(ptr[-1]), device=indptr.device)
    owner = torch.repeat_interleave(torch.arange(rows.numel(), device=indptr.device), lens)
    sel = keep[pos]
    counts = torch.bincount(owner[sel], minlength=rows.numel())
    out_ptr = torch.zeros(rows.numel() + 1, dtype=torch.int64, device=indptr.device)
    torch.cumsum(counts, 0, out=out_ptr[1:])
    return out_ptr, indices[pos[sel]].contiguous()


def holdout_split(indptr: torch.Tensor, indices: torch.Tensor, seed: int, test_fraction: float = 0.1,
                  heldout_fraction: float = 0.25):
    """Row split in the manner of the paper's Section 5 (strong generalisation): a hashed `test_fraction` of
    the rows are test rows and leave the training matrix; of each test row's links a hashed
    `heldout_fraction` are held out (to be predicted), the others are given (to fold the row in).

    Returns a dict: train_rows, test_rows (int64 row ids), train = (indptr, indices) over the training rows
    in order, given and held = (indptr, indices) over the test rows in order.  Index plumbing only."""
    dev = indptr.device
    m = indptr.numel() - 1
    r = torch.arange(m, device=dev, dtype=torch.int64)
    is_test = uniform01(hash_u64(seed, 21, r)) < test_fraction
    test_rows, train_rows = torch.nonzero(is_test).flatten(), torch.nonzero(~is_test).flatten()
    owner = _expand_rows(indptr)
    held = uniform01(hash_u64(seed, 23, owner, indices.to(torch.int64))) < heldout_fraction
    everything = torch.ones_like(held)
    return {
        "train_rows": train_rows, "test_rows": test_rows,
        "train": _select_entries(indptr, indices, train_rows, everything),
        "given": _select_entries(indptr, indices, test_rows, ~held),
        "held": _select_entries(indptr, indices, test_rows, held),
    }


def extract_rows(indptr: torch.Tensor, indices: torch.Tensor, values: Optional[torch.Tensor], rows: torch.Tensor):
    """Sub-matrix made of the listed rows, with its column ids renumbered densely.

    Returns (sub_indptr, sub_indices, sub_values, used_cols): row r of the result is row ``rows[r]``
    of the input and refers to column ``used_cols[sub_indices[p]]``.  Pure index plumbing, used to
    hand a sample of a large problem (and only the table rows it touches) to the CPU.
    """
    rows = rows.to(torch.int64)
    starts, lens = indptr[rows], indptr[rows + 1] - indptr[rows]
    sub_ptr = torch.zeros(rows.numel() + 1, dtype=torch.int64, device=indptr.device)
    torch.cumsum(lens, 0, out=sub_ptr[1:])
    total = int(sub_ptr[-1])
    pos = torch.repeat_interleave(starts - sub_ptr[:-1], lens) + torch.arange(total, device=indptr.device)
    used, inv = torch.unique(indices[pos], return_inverse=True)
    vals = None if values is None else values[pos].contiguous()
    return sub_ptr, inv.to(torch.int32).contiguous(), vals, used.to(torch.int64)
