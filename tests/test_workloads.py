"""The seeded input generators: shapes, determinism, NumPy/torch agreement."""
import numpy as np
import pytest
import torch

from paper_1205_2958_amd import workloads as W


def test_rows_are_sorted_distinct_and_in_range():
    nnz = np.array([0, 1, 5, 4096, 17, 0, 300], dtype=np.int64)
    for D in (1 << 12, 1 << 24, 1 << 30):
        col = W.csr_indices_np(nnz, D, seed=5)
        rp = W.row_ptr_from_nnz(nnz)
        assert col.dtype == np.uint32 and col.shape[0] == nnz.sum()
        for i in range(len(nnz)):
            r = col[rp[i]:rp[i + 1]].astype(np.int64)
            assert np.all(np.diff(r) > 0)
            assert r.size == 0 or (r[0] >= 0 and r[-1] < D)


def test_full_row_is_a_permutation_of_the_universe():
    D = 1 << 10
    col = W.csr_indices_np(np.array([D], dtype=np.int64), D, seed=9)
    assert np.array_equal(col, np.arange(D, dtype=np.uint32))


def test_indices_are_spread_uniformly():
    nnz = np.full(200, 2000, dtype=np.int64)
    col = W.csr_indices_np(nnz, 1 << 24, seed=77)
    hist = np.bincount(col >> 18, minlength=64).astype(np.float64)
    expect = hist.sum() / 64
    chi2 = ((hist - expect) ** 2 / expect).sum()
    assert chi2 < 130.0          # 63 degrees of freedom; 130 is far in the tail


def test_rows_differ_and_seed_matters():
    nnz = np.full(3, 50, dtype=np.int64)
    a = W.csr_indices_np(nnz, 1 << 24, seed=1).reshape(3, 50)
    b = W.csr_indices_np(nnz, 1 << 24, seed=2).reshape(3, 50)
    assert not np.array_equal(a[0], a[1]) and not np.array_equal(a, b)
    assert np.array_equal(a, W.csr_indices_np(nnz, 1 << 24, seed=1).reshape(3, 50))
    # a slice of rows generated on its own equals the same rows of the whole
    tail = W.csr_indices_np(nnz[1:], 1 << 24, seed=1, row_offset=1).reshape(2, 50)
    assert np.array_equal(tail, a[1:])


@pytest.mark.parametrize("D", [1 << 24, 1 << 30])
def test_torch_generator_matches_numpy(D):
    nnz = W.lognormal_nnz(300, 400.0, 1.0, 1, 5000, seed=3)
    nnz[5] = 0
    ref = W.csr_indices_np(nnz, D, seed=1234)
    got = W.csr_indices_torch(nnz, D, 1234, torch.device("cpu"), rows_per_block=64)
    assert np.array_equal(got.numpy().view(np.uint32), ref)


def test_workload_shapes_follow_the_dataset_table():
    w = W.WORKLOADS["large_2u"]
    nnz = w.nnz()
    assert nnz.shape == (350_000,) and nnz.min() >= 1 and nnz.max() <= 50_000
    assert 3600 < nnz.mean() < 3800                     # webspam: 3 728 nonzeros on average
    w5 = W.WORKLOADS["huge_2u_m61"]
    n5 = w5.nnz(batch=0)
    assert n5.shape == (200_000,) and n5.max() <= 1_000_000
    assert 8_000 < n5.mean() < 12_500                   # expanded rcv1: about 12 000
    assert w5.n_batches() == 10 and w5.sig_bytes() == 63
    assert W.WORKLOADS["perm_table"].sig_bytes() == 100


def test_coefficients_and_permutations():
    for fam in (W.FAMILY_2U_M31, W.FAMILY_4U_M31, W.FAMILY_2U_M61):
        c = W.coefficients(500, fam, seed=4)
        assert c.shape == (500, W.family_degree(fam)) and c.dtype == np.uint64
        assert int(c.max()) < W.family_prime(fam)
        assert int(c.max()) > W.family_prime(fam) // 2
    t = W.perm_table_np(256, 5, seed=6, perm_ld=8)
    assert t.shape == (256, 8)
    for j in range(5):
        assert np.array_equal(np.sort(t[:, j]), np.arange(256, dtype=np.uint32))
    # storage arithmetic of Section 2: D = 2^30, k = 500, 4 bytes each exceeds 2000 GB
    assert (1 << 30) * 500 * 4 > 2000 * 10 ** 9


def test_planted_pairs_have_the_stated_resemblance():
    rp, col, f1, f2 = W.planted_pairs(5, 1 << 16, union=400, shared=100, seed=8)
    for i in range(5):
        s1 = set(col[rp[2 * i]:rp[2 * i + 1]].tolist())
        s2 = set(col[rp[2 * i + 1]:rp[2 * i + 2]].tolist())
        assert len(s1) == f1 and len(s2) == f2
        assert len(s1 & s2) == 100 and len(s1 | s2) == 400


def test_stratified_rows_cover_the_named_rows_every_decile_and_the_budget():
    w = W.WORKLOADS["large_2u"]
    nnz = w.nnz(0)[:60_000]
    k, budget = 500, 2.0e9
    rows, cover = W.stratified_rows(nnz, k, budget, seed=1)
    again, _ = W.stratified_rows(nnz, k, budget, seed=1)
    assert np.array_equal(rows, again)                                   # seeded
    assert len(set(rows.tolist())) == len(rows) and np.all(np.diff(rows) > 0)
    spent = float(nnz[rows].sum()) * k
    assert spent <= budget and spent > 0.9 * budget
    assert cover["rows"] == len(rows) and cover["nonzeros"] == int(nnz[rows].sum())
    assert abs(cover["pct_of_evaluations"] - 100.0 * spent / (float(nnz.sum()) * k)) < 1e-9
    order = np.argsort(nnz, kind="stable")
    for r in (0, len(nnz) - 1, int(order[0]), int(order[-1])):
        assert r in rows
    # both neighbours of the split point and of its double
    lens = np.sort(nnz[rows])
    for m in (8192, 16384):
        assert lens[np.searchsorted(lens, m, side="right") - 1] == nnz[nnz <= m].max()
        assert lens[np.searchsorted(lens, m, side="right")] == nnz[nnz > m].min()
    # every decile of the length distribution is represented
    edges = np.quantile(nnz, np.linspace(0, 1, 11))
    hist, _ = np.histogram(nnz[rows], bins=edges)
    assert np.all(hist > 0)
    # a cap on the cost of one row keeps longer rows out; heavy rows are taken first when asked for
    rows2, cover2 = W.stratified_rows(nnz, k, budget, seed=1, max_row_evals=20_000 * k, heavy_from=15_000)
    assert nnz[rows2].max() <= 20_000 and cover2["longest_row"] == nnz[nnz <= 20_000].max()
    assert (nnz[rows2] >= 15_000).sum() > (nnz[rows] >= 15_000).sum()
    # everything fits: every row is taken
    small = nnz[:50]
    all_rows, cover3 = W.stratified_rows(small, k, 1e15, seed=2)
    assert np.array_equal(all_rows, np.arange(50)) and cover3["pct_of_evaluations"] == 100.0


def test_rows_can_be_generated_one_by_one_by_number():
    nnz = np.array([7, 0, 300, 12], dtype=np.int64)
    whole = W.csr_indices_np(nnz, 1 << 16, seed=9)
    rp = W.row_ptr_from_nnz(nnz)
    pick = np.array([2, 0, 3])
    got = W.csr_indices_np(nnz[pick], 1 << 16, seed=9, rows=pick)
    want = np.concatenate([whole[rp[r]:rp[r + 1]] for r in pick])
    assert np.array_equal(got, want)
