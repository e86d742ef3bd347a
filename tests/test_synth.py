"""Host checks of the seeded input generators (no method arithmetic involved)."""
import numpy as np
import torch

from synth import hash_u64, init_table, make_problem, uniform01
from synth.matrices import _mix  # noqa: F401  (import check)

M64 = (1 << 64) - 1


def _ref_mix(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def _ref_hash(seed, stream, a, b):
    k = ((seed * 0x9E3779B97F4A7C15) ^ (stream * 0xD6E8FEB86659FD93)) & M64
    z = _ref_mix((a * 0x9E3779B97F4A7C15 + k) & M64)
    return _ref_mix(z ^ ((b * 0xD6E8FEB86659FD93 + 0x9E3779B97F4A7C15) & M64))


def test_hash_matches_pure_python_unsigned_reference():
    a = torch.tensor([0, 1, 2, 12345678901, 2**40 + 7], dtype=torch.int64)
    for b in (0, 5, 999):
        got = hash_u64(77, 3, a, torch.full_like(a, b))
        got_scalar_b = hash_u64(77, 3, a, b)
        for x, g, g2 in zip(a.tolist(), got.tolist(), got_scalar_b.tolist()):
            ref = _ref_hash(77, 3, x, b)
            assert (g & M64) == ref and (g2 & M64) == ref


def test_uniform_is_open_interval_and_flat():
    u = uniform01(hash_u64(1, 2, torch.arange(200000)))
    assert float(u.min()) > 0.0 and float(u.max()) < 1.0
    hist = torch.histc(u, bins=10, min=0, max=1) / u.numel()
    assert float((hist - 0.1).abs().max()) < 0.005


def test_init_table_scale():
    T = init_table(20000, 16, seed=5, stream=11)
    assert T.dtype == torch.float32 and T.shape == (20000, 16)
    assert abs(float(T.double().std()) - 0.1 / 4.0) < 5e-4
    assert torch.equal(T, init_table(20000, 16, seed=5, stream=11, chunk=777))


def _check_csr(rows, cols, indptr, indices):
    ip, ix = indptr.numpy(), indices.numpy()
    assert ip.dtype == np.int64 and ix.dtype == np.int32
    assert ip[0] == 0 and ip[-1] == ix.size and np.all(np.diff(ip) >= 0) and ip.size == rows + 1
    assert ix.min() >= 0 and ix.max() < cols
    r = np.repeat(np.arange(rows), np.diff(ip))
    key = r.astype(np.int64) * cols + ix
    assert np.all(np.diff(key) > 0)  # sorted by (row, col) and no duplicate pair
    return set(zip(r.tolist(), ix.tolist()))


def test_c1_matrix_is_valid_and_transpose_is_true_transpose():
    p = make_problem("c1")
    assert (p.rows, p.cols, p.d) == (2000, 1500, 16)
    s = p.stats()
    assert 15 <= s["row_deg_mean"] <= 30 and s["row_deg_max"] <= 200
    e = _check_csr(p.rows, p.cols, p.indptr, p.indices)
    et = _check_csr(p.cols, p.rows, p.t_indptr, p.t_indices)
    assert {(c, r) for r, c in e} == et
    q = make_problem("c1")
    assert torch.equal(p.indices, q.indices) and torch.equal(p.W0, q.W0)


def test_scaled_down_recipes_have_the_stated_shape():
    for kind, mean_lo, mean_hi in (("c2", 27, 33), ("c3", 14, 21), ("c4", 5.5, 6.5), ("c5", 22, 28)):
        p = make_problem(kind, rows=30000, cols=30000, d=8)
        s = p.stats()
        _check_csr(p.rows, p.cols, p.indptr, p.indices)
        assert mean_lo <= s["row_deg_mean"] <= mean_hi, (kind, s)
    p = make_problem("c3", rows=30000, cols=30000, d=8)
    assert p.stats()["col_deg_max"] > 1000  # popular targets form hubs on the column side


def test_values_option_and_transpose_carries_values():
    p = make_problem("c1", rows=120, cols=90, values="uniform")
    assert p.values.dtype == torch.float32 and float(p.values.min()) >= 0.5 and float(p.values.max()) < 1.5
    r = np.repeat(np.arange(p.rows), np.diff(p.indptr.numpy()))
    fwd = {(a, b): v for a, b, v in zip(r.tolist(), p.indices.tolist(), p.values.tolist())}
    rt = np.repeat(np.arange(p.cols), np.diff(p.t_indptr.numpy()))
    bwd = {(b, a): v for a, b, v in zip(rt.tolist(), p.t_indices.tolist(), p.t_values.tolist())}
    assert fwd == bwd


def test_extract_rows_is_a_faithful_submatrix():
    from synth import extract_rows
    p = make_problem("c1", rows=300, cols=250, values="uniform")
    pick = torch.tensor([7, 0, 299, 41, 41])
    sp, si, sv, used = extract_rows(p.indptr, p.indices, p.values, pick)
    assert sp[0] == 0 and sp.numel() == 6
    for r, u in enumerate(pick.tolist()):
        a, b = int(p.indptr[u]), int(p.indptr[u + 1])
        assert torch.equal(used[si[sp[r]:sp[r + 1]].long()], p.indices[a:b].long())
        assert torch.equal(sv[sp[r]:sp[r + 1]], p.values[a:b])


def test_block_size_does_not_change_the_matrix_and_degrees_are_the_drawn_ones():
    """Row blocks and column ranges are plumbing: any block size gives the same CSR and the same transpose;
    with redrawn collisions every row holds exactly its drawn number of distinct column ids."""
    from synth.matrices import CONFIGS, _degrees, build_csr, transpose_csr
    n = 20000
    for kind in ("c2", "c3", "c4", "c5"):
        seed = CONFIGS[kind]["seed"]
        deg = torch.clamp(_degrees(kind, n, seed, "cpu"), max=n - 1)
        big = build_csr(kind, n, n, seed, deg)
        small = build_csr(kind, n, n, seed, deg, block=30011)
        assert torch.equal(big[0], small[0]) and torch.equal(big[1], small[1])
        assert torch.equal(big[0][1:] - big[0][:-1], deg)
        _check_csr(n, n, big[0], big[1])
        ta = transpose_csr(n, n, big[0], big[1])
        tb = transpose_csr(n, n, big[0], big[1], block=30011)
        assert torch.equal(ta[0], tb[0]) and torch.equal(ta[1], tb[1])
        _check_csr(n, n, ta[0], ta[1])


def test_transpose_with_values_in_column_ranges():
    from synth.matrices import transpose_csr
    p = make_problem("c1", rows=300, cols=250, values="uniform")
    a = transpose_csr(p.rows, p.cols, p.indptr, p.indices, p.values)
    b = transpose_csr(p.rows, p.cols, p.indptr, p.indices, p.values, block=97)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert torch.equal(a[2], p.t_values) and torch.equal(a[1], p.t_indices)
