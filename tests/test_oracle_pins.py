"""Pins for the CPU oracle: it is checked against things other than itself.

Each test states what it pins.  References: the objective is Eq. 3 of the paper
(Section 3), the row update is Eq. 4, the loop structure is Algorithm 1.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from synth import make_problem

RNG = np.random.default_rng(1234)


def random_problem(m, n, d, density=0.3, general_y=True, rng=RNG, empty_row=True):
    mask = rng.random((m, n)) < density
    if empty_row and m > 1:
        mask[1, :] = False  # one row with no observed entry
    indptr = np.zeros(m + 1, dtype=np.int64)
    indptr[1:] = np.cumsum(mask.sum(1))
    indices = np.concatenate([np.nonzero(mask[u])[0] for u in range(m)]).astype(np.int32)
    values = (rng.random(indices.size) + 0.5).astype(np.float32) if general_y else None
    H = rng.normal(0, 0.5, (n, d))
    return indptr, indices, values, H


def dense_lstsq_rows(indptr, indices, values, H, alpha, lam):
    """Eq. 3 restricted to one row is a linear least-squares problem: stack the
    observed rows of H, sqrt(alpha) * all of H, and sqrt(lam) * I; targets y, 0, 0."""
    m = indptr.size - 1
    n, d = H.shape
    out = np.zeros((m, d))
    for u in range(m):
        idx = indices[indptr[u]:indptr[u + 1]]
        y = np.ones(idx.size) if values is None else values[indptr[u]:indptr[u + 1]].astype(np.float64)
        X = np.vstack([H[idx], np.sqrt(alpha) * H, np.sqrt(lam) * np.eye(d)])
        t = np.concatenate([y, np.zeros(n), np.zeros(d)])
        out[u] = np.linalg.lstsq(X, t, rcond=None)[0]
    return out


@pytest.mark.parametrize("m,n,d,alpha,lam", [(30, 40, 8, 0.1, 1e-2), (50, 20, 5, 0.7, 0.3), (12, 50, 3, 0.01, 1e-3)])
@pytest.mark.parametrize("general_y", [False, True])
def test_matches_bruteforce_least_squares(m, n, d, alpha, lam, general_y):
    indptr, indices, values, H = random_problem(m, n, d, general_y=general_y)
    X = oracle.half_epoch(indptr, indices, values, H, alpha, lam)
    ref = dense_lstsq_rows(indptr, indices, values, H, alpha, lam)
    assert np.linalg.norm(X - ref) <= 1e-9 * np.linalg.norm(ref)


def test_matches_bruteforce_on_c1_shaped_input():
    p = make_problem("c1", rows=200, cols=150)
    H = p.H0.double().numpy() * 10.0
    ip, ix = p.indptr.numpy(), p.indices.numpy()
    X = oracle.half_epoch(ip, ix, None, H, p.alpha, p.lam)
    ref = dense_lstsq_rows(ip, ix, None, H, p.alpha, p.lam)
    assert np.linalg.norm(X - ref) <= 1e-9 * np.linalg.norm(ref)


def test_zero_gradient_with_literal_all_pairs_sum():
    """d/dw of Eq. 3 vanishes at the solution; the alpha term is summed over all n items."""
    alpha, lam = 0.2, 0.05
    indptr, indices, values, H = random_problem(25, 35, 6)
    X = oracle.half_epoch(indptr, indices, values, H, alpha, lam)
    for u in range(25):
        w = X[u]
        sl = slice(indptr[u], indptr[u + 1])
        g = lam * w
        for i in range(H.shape[0]):
            g = g + alpha * H[i] * (H[i] @ w)
        b = np.zeros_like(w)
        for i, y in zip(indices[sl], values[sl]):
            g = g + H[i] * (H[i] @ w) - float(y) * H[i]
            b += float(y) * H[i]
        assert np.linalg.norm(g) <= 1e-10 * max(np.linalg.norm(b), 1e-30)


def test_objective_never_increases_on_c1():
    """Exact block minimisation: Eq. 3 (literal double sum) is non-increasing over 8 half-epochs."""
    p = make_problem("c1")
    Y = (p.indptr.numpy(), p.indices.numpy(), None)
    Yt = (p.t_indptr.numpy(), p.t_indices.numpy(), None)
    W, H = p.W0.double().numpy(), p.H0.double().numpy()
    losses = [oracle.loss(Y, W, H, p.alpha, p.lam, literal=True)]
    for _ in range(p.epochs):
        W = oracle.half_epoch(*Y, H, p.alpha, p.lam)
        losses.append(oracle.loss(Y, W, H, p.alpha, p.lam, literal=True))
        H = oracle.half_epoch(*Yt, W, p.alpha, p.lam)
        losses.append(oracle.loss(Y, W, H, p.alpha, p.lam, literal=True))
    for a, b in zip(losses, losses[1:]):
        assert b <= a * (1 + 1e-12)
    assert losses[-1] < 0.9 * losses[0]
    # the two-half epoch entry point walks the same path
    W2, H2 = p.W0.double().numpy(), p.H0.double().numpy()
    for _ in range(p.epochs):
        W2, H2 = oracle.epoch(Y, Yt, W2, H2, p.alpha, p.lam)
    assert np.array_equal(W2, W) and np.array_equal(H2, H)


def test_closed_form_empty_row_is_zero():
    indptr, indices, values, H = random_problem(10, 12, 4)
    X = oracle.half_epoch(indptr, indices, values, H, 0.3, 0.1)
    assert indptr[2] == indptr[1] and np.all(X[1] == 0.0)


def test_closed_form_single_entry_sherman_morrison():
    alpha, lam = 0.15, 0.02
    n, d = 20, 6
    H = RNG.normal(0, 1, (n, d))
    indptr = np.arange(n + 1, dtype=np.int64)
    indices = RNG.permutation(n).astype(np.int32)
    values = (RNG.random(n) + 0.5).astype(np.float32)
    X = oracle.half_epoch(indptr, indices, values, H, alpha, lam)
    B = alpha * H.T @ H + lam * np.eye(d)
    for u in range(n):
        h, y = H[indices[u]], float(values[u])
        Bih = np.linalg.solve(B, h)
        w = y * Bih / (1.0 + h @ Bih)
        assert np.allclose(X[u], w, rtol=1e-11, atol=1e-14)


def test_closed_form_d_equals_one():
    alpha, lam = 0.4, 0.03
    indptr, indices, values, H = random_problem(15, 25, 1)
    X = oracle.half_epoch(indptr, indices, values, H, alpha, lam)
    tot = float((H[:, 0] ** 2).sum())
    for u in range(15):
        sl = slice(indptr[u], indptr[u + 1])
        h = H[indices[sl], 0]
        w = (values[sl].astype(np.float64) * h).sum() / ((h ** 2).sum() + alpha * tot + lam)
        assert abs(X[u, 0] - w) <= 1e-13 * max(1.0, abs(w))


def test_closed_form_identity_table():
    alpha, lam = 0.25, 0.5
    d = 7
    indptr, indices, values, _ = random_problem(9, d, d, density=0.5)
    X = oracle.half_epoch(indptr, indices, values, np.eye(d), alpha, lam)
    ref = np.zeros((9, d))
    for u in range(9):
        sl = slice(indptr[u], indptr[u + 1])
        ref[u, indices[sl]] = values[sl].astype(np.float64) / (1.0 + alpha + lam)
    assert np.allclose(X, ref, rtol=1e-13, atol=1e-15)


def test_closed_form_alpha_zero_is_ridge_regression():
    lam = 0.07
    indptr, indices, values, H = random_problem(20, 30, 5)
    X = oracle.half_epoch(indptr, indices, values, H, 0.0, lam)
    for u in range(20):
        sl = slice(indptr[u], indptr[u + 1])
        Hs, y = H[indices[sl]], values[sl].astype(np.float64)
        w = np.linalg.lstsq(np.vstack([Hs, np.sqrt(lam) * np.eye(5)]),
                            np.concatenate([y, np.zeros(5)]), rcond=None)[0]
        assert np.allclose(X[u], w, rtol=1e-9, atol=1e-12)


def test_gramian_invariants_and_library_matmul():
    V = RNG.normal(0, 1, (300, 9))
    G = oracle.gramian(V)
    assert np.array_equal(G, G.T)
    assert np.linalg.eigvalsh(G).min() > 0
    assert np.isclose(np.trace(G), (V ** 2).sum(), rtol=1e-13)
    assert np.allclose(G, V.T @ V, rtol=1e-12, atol=1e-12)
    # a non-symmetric construction: asymmetric V catches a transposed operand
    V2 = np.zeros((2, 3)); V2[0] = [1, 2, 3]; V2[1] = [0, 1, 0]
    assert np.array_equal(oracle.gramian(V2), np.array([[1, 2, 3], [2, 5, 6], [3, 6, 9.0]]))


def test_matmul_gramian_equals_plain_loop_gramian():
    V = RNG.normal(0, 1, (5000, 12)).astype(np.float32)
    a, b = oracle.gramian(V), oracle.gramian_matmul(V, chunk=777)
    assert np.abs(a - b).max() <= 1e-11 * np.abs(a).max()


def test_solution_is_linear_in_labels_and_order_free():
    alpha, lam = 0.1, 0.01
    indptr, indices, values, H = random_problem(12, 30, 6)
    X = oracle.half_epoch(indptr, indices, values, H, alpha, lam)
    X3 = oracle.half_epoch(indptr, indices, 4.0 * values, H, alpha, lam)  # x4 is exact in fp32
    assert np.allclose(X3, 4.0 * X, rtol=1e-12, atol=1e-14)
    # reverse the entries inside every row: same set, same solution up to summation order
    ridx, rval = indices.copy(), values.copy()
    for u in range(12):
        sl = slice(indptr[u], indptr[u + 1])
        ridx[sl], rval[sl] = indices[sl][::-1], values[sl][::-1]
    assert np.allclose(oracle.half_epoch(indptr, ridx, rval, H, alpha, lam), X, rtol=1e-11, atol=1e-14)
    # row subset / row order: rows are independent given (V, G)
    G = oracle.gramian(H)
    pick = np.array([7, 0, 3], dtype=np.int64)
    assert np.array_equal(oracle.solve_rows(indptr, indices, values, H, G, alpha, lam, pick), X[pick])


def test_loss_trace_form_equals_literal_double_sum():
    indptr, indices, values, H = random_problem(17, 23, 5)
    W = RNG.normal(0, 0.7, (17, 5))
    Y = (indptr, indices, values)
    a = oracle.loss(Y, W, H, 0.3, 0.02, literal=False)
    b = oracle.loss(Y, W, H, 0.3, 0.02, literal=True)
    assert abs(a - b) <= 1e-12 * abs(b)
    # and against the objective typed out densely with numpy
    P = W @ H.T
    dense = 0.3 * (P ** 2).sum() + 0.02 * ((W ** 2).sum() + (H ** 2).sum())
    for u in range(17):
        for p in range(indptr[u], indptr[u + 1]):
            dense += (float(values[p]) - P[u, indices[p]]) ** 2
    assert abs(b - dense) <= 1e-12 * abs(dense)


def test_exact_rational_fixture():
    """A 3x4, d=2 problem solved in exact rational arithmetic (Gaussian elimination on
    fractions; tests/golden/make_tiny_rational.py).  Pins Eq. 4 and Eq. 3 end to end."""
    with open(os.path.join(os.path.dirname(__file__), "golden", "tiny_rational.json")) as f:
        g = json.load(f)
    Y = (np.array(g["indptr"]), np.array(g["indices"]), np.array(g["values"], dtype=np.float32))
    H = np.array(g["H"], dtype=np.float64)
    X = oracle.half_epoch(*Y, H, g["alpha"], g["lambda"])
    assert np.allclose(X, np.array(g["W_solved"]), rtol=1e-13, atol=1e-15)
    L = oracle.loss(Y, X, H, g["alpha"], g["lambda"])
    assert abs(L - g["loss_at_solution"]) <= 1e-12 * abs(g["loss_at_solution"])


def test_storage_rounding_matches_library_casts():
    x = np.concatenate([RNG.normal(0, 1, 4000), RNG.normal(0, 1e-3, 4000), [0.0, 1.0, -1.0, 1.00390625, 1.01171875]])
    t = torch.from_numpy(x)
    assert np.array_equal(oracle.round_storage(x, "f32"), t.float().double().numpy())
    assert np.array_equal(oracle.round_storage(x, "bf16"), t.float().bfloat16().double().numpy())
    assert np.array_equal(oracle.round_storage(x, "f64"), x)
    X = oracle.half_epoch(*random_problem(6, 9, 4)[:3], RNG.normal(0, 1, (9, 4)), 0.1, 0.01, storage="bf16")
    assert np.array_equal(X, torch.from_numpy(X).bfloat16().double().numpy())


def test_topk_and_recall_against_brute_force():
    """oracle.topk / recall_at_k pinned to a pure-Python evaluation on tiny inputs: every score by a literal
    dot product, candidates sorted as (-score, id) tuples, exclusions removed, including exact ties."""
    rng = np.random.default_rng(11)
    Q = rng.integers(-3, 4, size=(7, 5)).astype(np.float64)   # small integers: many exactly equal scores
    H = rng.integers(-3, 4, size=(23, 5)).astype(np.float64)
    ex_ptr = np.array([0, 0, 3, 3, 10, 10, 11, 11 + 22], dtype=np.int64)
    ex_idx = np.concatenate([[4, 9, 0], np.arange(3, 10), [22], np.arange(22)]).astype(np.int32)
    for k in (1, 4, 23, 30):
        ids, sc = oracle.topk(Q, H, k, (ex_ptr, ex_idx))
        for q in range(7):
            banned = set(ex_idx[ex_ptr[q]:ex_ptr[q + 1]].tolist())
            cand = sorted((-sum(Q[q, c] * H[i, c] for c in range(5)), i) for i in range(23) if i not in banned)
            want = [i for _, i in cand[:k]] + [-1] * max(0, k - len(cand))
            assert ids[q].tolist() == want
            assert all(sc[q, r] == -cand[r][0] for r in range(min(k, len(cand))))
    ids, _ = oracle.topk(Q, H, 4)
    held_ptr = np.array([0, 2, 2, 3, 4, 5, 6, 12], dtype=np.int64)
    held_idx = np.array([ids[0, 0], ids[0, 3], ids[2, 1], 99, ids[4, 2], 99, *ids[6, :4], 97, 98], dtype=np.int64)
    rec = oracle.recall_at_k(ids, held_ptr, held_idx)
    assert rec[0] == 1.0 and np.isnan(rec[1]) and rec[2] == 1.0 and rec[3] == 0.0 and rec[4] == 1.0 and rec[5] == 0.0
    assert rec[6] == 1.0  # six held-out links, four of them retrieved: 4 / min(4, 6)
