"""GPU parity of the evaluation path on synthetic data: fold-in of held-out rows with Eq. 4 (Section 5 of the
paper: a test row is embedded from 75% of its links with the item table fixed) and exact top-k retrieval
(Section 4.6), with Recall@20 / Recall@50 computed from the retrieved ids.  No item of the paper's dataset is
involved: the matrix is the synthetic host-locality recipe, split by hashed row and link.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import f64, max_row_err, rel_fro, say
from paper_2112_02194_amd import binding as als
from synth import holdout_split, init_table, make_problem, transpose_csr

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(gpu_device):
    c = als.Context(0)
    yield c
    c.close()


def _check_topk(ids, sc, Qh, Hh, k, exclude, tol):
    """GPU top-k against the fp64 definition: what is unique is compared exactly, the rest is checked to be valid."""
    ref_ids, ref_sc = oracle.topk(Qh, Hh, k, exclude)
    S = Qh @ Hh.T
    scale = np.abs(S).max()
    exact = 0
    for q in range(Qh.shape[0]):
        got = ids[q]
        n_ok = int((ref_ids[q] >= 0).sum())
        assert np.all(got[n_ok:] == -1) and np.all(np.isneginf(sc[q, n_ok:]))
        got = got[:n_ok]
        assert len(set(got.tolist())) == n_ok and got.min(initial=0) >= 0
        if exclude is not None:
            banned = exclude[1][exclude[0][q]:exclude[0][q + 1]]
            assert not np.intersect1d(got, banned).size
        assert np.all(np.abs(sc[q, :n_ok] - S[q, got]) <= tol * scale)        # the scores are those of the ids
        assert np.all(np.diff(sc[q, :n_ok]) <= 0)                               # best first
        assert np.all(np.abs(sc[q, :n_ok] - ref_sc[q, :n_ok]) <= tol * scale)  # rank by rank the same score
        gaps = np.abs(np.diff(np.sort(S[q][np.isfinite(S[q])])[::-1][:n_ok + 1]))
        if gaps.size == 0 or gaps.min() > 4 * tol * scale:                      # no near-tie: the ranking is unique
            assert np.array_equal(got, ref_ids[q, :n_ok])
            exact += 1
    return exact


@pytest.mark.parametrize("d,dtype,k", [(128, torch.float32, 50), (32, torch.float32, 20), (64, torch.bfloat16, 64),
                                       (16, torch.float32, 1), (128, torch.bfloat16, 7)])
def test_topk_matches_the_definition(ctx, gpu_device, d, dtype, k):
    say(f"als_topk d={d} {dtype} k={k}")
    nq, n = 333, 20011  # ragged: not multiples of 16 or 64; three slices of the item table
    Q = (init_table(nq, d, seed=31, stream=5) * 10).to(dtype)
    H = (init_table(n, d, seed=31, stream=7) * 10).to(dtype)
    H[100:140] = H[99]  # forty identical items: exact ties, broken by id
    gen = torch.Generator().manual_seed(3)
    lens = torch.randint(0, 40, (nq,), generator=gen)
    lens[5] = 0
    ex_ptr = torch.zeros(nq + 1, dtype=torch.int64)
    ex_ptr[1:] = torch.cumsum(lens, 0)
    ex_idx = torch.cat([torch.randperm(n, generator=gen)[:int(l)] for l in lens]).to(torch.int32)
    ex = als.Csr(nq, n, ex_ptr.to(gpu_device), ex_idx.to(gpu_device))
    for exclude in (None, ex):
        ids, sc = als.als_topk(ctx, Q.to(gpu_device), H.to(gpu_device), k, exclude)
        torch.cuda.synchronize()
        exh = None if exclude is None else (ex_ptr.numpy(), ex_idx.numpy())
        exact = _check_topk(ids.cpu().numpy(), sc.cpu().numpy(), f64(Q), f64(H), k, exh, 2e-6)
        say(f"  exclude={exclude is not None}: {exact} of {nq} rankings unique and identical")
        assert exact > nq // 2 or k > 40


def test_topk_with_fewer_admissible_items_than_k(ctx, gpu_device):
    say("als_topk: tiny item table, everything excluded for one query")
    Q, H = init_table(3, 32, seed=1, stream=1) * 10, init_table(10, 32, seed=1, stream=2) * 10
    ex_ptr = torch.tensor([0, 10, 10, 14], dtype=torch.int64)
    ex_idx = torch.cat([torch.arange(10), torch.tensor([1, 3, 5, 7])]).to(torch.int32)
    ex = als.Csr(3, 10, ex_ptr.to(gpu_device), ex_idx.to(gpu_device))
    ids, sc = als.als_topk(ctx, Q.to(gpu_device), H.to(gpu_device), 16, ex)
    torch.cuda.synchronize()
    _check_topk(ids.cpu().numpy(), sc.cpu().numpy(), f64(Q), f64(H), 16, (ex_ptr.numpy(), ex_idx.numpy()), 2e-6)
    assert torch.all(ids[0] == -1) and int((ids[1] >= 0).sum()) == 10 and int((ids[2] >= 0).sum()) == 6
    with pytest.raises(als.AlsError):
        als.als_topk(ctx, Q.to(gpu_device), H.to(gpu_device), 65)


def test_fold_in_and_recall_follow_the_oracle(ctx, gpu_device):
    """Section 5 protocol on a synthetic link matrix: 90/10 row split, two epochs on the training rows, test rows
    folded in from 75% of their links (Eq. 4 with the item table fixed), top-50 retrieval without the given
    links, Recall@20 and Recall@50 on the held-out 25%."""
    say("fold-in + top-k + Recall@K, 30000 nodes, d = 64")
    p = make_problem("c3", rows=30000, cols=30000, d=64)
    sp = holdout_split(p.indptr, p.indices, seed=99)
    tr_ptr, tr_idx = sp["train"]
    n_train, n_test, n = sp["train_rows"].numel(), sp["test_rows"].numel(), p.cols
    assert 0.08 * p.rows < n_test < 0.12 * p.rows
    tt_ptr, tt_idx, _ = transpose_csr(n_train, n, tr_ptr, tr_idx)
    dev = gpu_device
    Y, Yt = als.Csr(n_train, n, tr_ptr.to(dev), tr_idx.to(dev)), als.Csr(n, n_train, tt_ptr.to(dev), tt_idx.to(dev))
    W0, H0 = p.W0[sp["train_rows"]].contiguous(), p.H0
    W, H = W0.to(dev), H0.to(dev)
    prm = als.make_params(p.alpha, p.lam)
    Wo, Ho = f64(W0), f64(H0)
    for _ in range(2):
        als.als_epoch(ctx, Y, Yt, W, H, prm)
        Wo, Ho = oracle.epoch((tr_ptr.numpy(), tr_idx.numpy(), None), (tt_ptr.numpy(), tt_idx.numpy(), None), Wo, Ho,
                              p.alpha, p.lam, storage="f32")
    assert rel_fro(f64(H), Ho) <= 1e-4
    # fold-in: Eq. 4 for the test rows from their given links, item table and its Gramian fixed
    gv_ptr, gv_idx = sp["given"]
    G = als.als_gramian(ctx, H)
    Yg = als.Csr(n_test, n, gv_ptr.to(dev), gv_idx.to(dev))
    Xt = torch.zeros(n_test, p.d, device=dev)
    als.als_solve_rows(ctx, Yg, H, G, prm, Xt)
    als.als_status_sync(ctx)
    Xo = oracle.solve_rows(gv_ptr.numpy(), gv_idx.numpy(), None, Ho, oracle.gramian(Ho), p.alpha, p.lam, None, "f32")
    say(f"  folded-in rows: rel err {rel_fro(f64(Xt), Xo):.2e}, worst row {max_row_err(f64(Xt), Xo):.2e}")
    assert rel_fro(f64(Xt), Xo) <= 1e-4 and max_row_err(f64(Xt), Xo) <= 1e-4
    # retrieval without the links the row was folded in from, and recall on the held-out ones
    ids, sc = als.als_topk(ctx, Xt, H, 50, Yg)
    torch.cuda.synchronize()
    ids = ids.cpu().numpy()
    sub = np.arange(0, n_test, 7)  # the definition is O(n_test * n): check a seventh of the test rows in full
    exh = (gv_ptr.numpy(), gv_idx.numpy())
    sub_ptr = np.concatenate([[0], np.cumsum(np.diff(exh[0])[sub])])
    sub_idx = np.concatenate([exh[1][exh[0][q]:exh[0][q + 1]] for q in sub])
    _check_topk(ids[sub], sc.cpu().numpy()[sub], f64(Xt)[sub], f64(H), 50, (sub_ptr, sub_idx), 2e-6)
    hd_ptr, hd_idx = sp["held"]
    ref_ids, _ = oracle.topk(Xo, Ho, 50, exh)
    for K in (20, 50):
        rg = np.nanmean(oracle.recall_at_k(ids[:, :K], hd_ptr.numpy(), hd_idx.numpy()))
        ro = np.nanmean(oracle.recall_at_k(ref_ids[:, :K], hd_ptr.numpy(), hd_idx.numpy()))
        say(f"  Recall@{K}: library {rg:.4f}, oracle {ro:.4f}")
        assert abs(rg - ro) <= 2e-3 and rg > 0.05  # far above chance (K / n = 0.002)
