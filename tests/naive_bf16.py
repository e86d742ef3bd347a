"""Test-only model of the failure the paper's Section 4.4 warns about: iALS with bfloat16 numerics used naively.

Every operand and every intermediate result - the Gramian's running sums, the per-row statistics, each step
of the Cholesky factorisation and of the two triangular solves - is rounded to bfloat16 (round to nearest
even), which is what "the whole update in bfloat16" means on a bfloat16 machine.  This is NOT a product path
and not the oracle of one: it exists so that the precision test can show, on the same synthetic inputs, that
this policy falls apart when the regulariser is small while the policy the paper settles on (bf16 storage,
fp32 arithmetic, one rounding on store; oracle storage="bf16" and the HIP library) does not.  Plain numpy,
batched over rows; a non-positive pivot yields NaN, as sqrt would.
"""
import numpy as np


def bf16(x):
    """Round fp32 values to the nearest bfloat16 (ties to even), returned as fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = ((u + (0x7FFF + ((u >> 16) & 1))) & 0xFFFF0000).astype(np.uint32)
    out = r.view(np.float32).copy()
    out[np.isnan(x)] = np.nan
    return out


def gramian(V):
    G = np.zeros((V.shape[1], V.shape[1]), dtype=np.float32)
    for j in range(V.shape[0]):
        G = bf16(G + bf16(np.outer(V[j], V[j])))
    return G


def half_epoch(indptr, indices, V, alpha, lam):
    """Eq. 4 for every row, all arithmetic rounded to bf16; V is a bf16-valued fp32 array."""
    m, d = indptr.size - 1, V.shape[1]
    deg = np.diff(indptr)
    A = np.broadcast_to(bf16(bf16(np.float32(alpha) * gramian(V)) + bf16(np.float32(lam) * np.eye(d, dtype=np.float32))),
                        (m, d, d)).copy()
    b = np.zeros((m, d), dtype=np.float32)
    for j in range(int(deg.max(initial=0))):  # the j-th stored entry of every row that has one
        rows = np.nonzero(deg > j)[0]
        h = V[indices[indptr[rows] + j]]
        A[rows] = bf16(A[rows] + bf16(h[:, :, None] * h[:, None, :]))
        b[rows] = bf16(b[rows] + h)  # y = 1
    with np.errstate(invalid="ignore", divide="ignore"):
        L = np.zeros_like(A)
        for c in range(d):  # Cholesky, column by column
            s = A[:, c, c].copy()
            for p in range(c):
                s = bf16(s - bf16(L[:, c, p] * L[:, c, p]))
            piv = bf16(np.sqrt(np.where(s > 0, s, np.nan)))
            L[:, c, c] = piv
            for r in range(c + 1, d):
                t = A[:, r, c].copy()
                for p in range(c):
                    t = bf16(t - bf16(L[:, r, p] * L[:, c, p]))
                L[:, r, c] = bf16(t / piv)
        z = np.zeros_like(b)
        for r in range(d):  # L z = b
            t = b[:, r].copy()
            for p in range(r):
                t = bf16(t - bf16(L[:, r, p] * z[:, p]))
            z[:, r] = bf16(t / L[:, r, r])
        x = np.zeros_like(b)
        for r in range(d - 1, -1, -1):  # L^T x = z
            t = z[:, r].copy()
            for p in range(r + 1, d):
                t = bf16(t - bf16(L[:, p, r] * x[:, p]))
            x[:, r] = bf16(t / L[:, r, r])
    x[deg == 0] = 0.0
    return x


def epoch(Y, Yt, W, H, alpha, lam):
    W = half_epoch(Y[0], Y[1], bf16(H), alpha, lam)
    H = half_epoch(Yt[0], Yt[1], W, alpha, lam)
    return W, H
