"""Host-side checks of the synthetic workload generators (shapes, structure, determinism)."""
import numpy as np

from paper_1708_04801_amd import workloads as wl


def test_tiny_hinge_full_size_matches_the_stated_recipe():
    w = wl.tiny_hinge()
    assert (w.m, w.d, w.k) == (4096, 64, 4) and w.loss == wl.HINGE
    assert w.n_steps.tolist() == [1000, 800, 600, 400] and (w.eta, w.lam, w.seed) == (0.01, 1e-3, 0)
    assert w.dense.dtype == np.float32 and w.dense.shape == (4096, 64)
    assert set(np.unique(w.y)) == {-1.0, 1.0}
    assert abs(w.dense.mean()) < 0.01 and abs(w.dense.std() - 1) < 0.01
    again = wl.tiny_hinge()
    assert np.array_equal(again.dense, w.dense) and np.array_equal(again.y, w.y)


def test_dense_logistic_small_instance():
    w = wl.dense_logistic(m=2048, d=512, k=8, n_lo=50, n_hi=200)
    assert w.dense.shape == (2048, 512) and w.loss == wl.LOGISTIC
    assert 50 <= w.n_steps.min() and w.n_steps.max() <= 200
    assert abs(w.dense.std() - 1 / np.sqrt(512)) < 1e-3
    assert 0.3 < (w.y > 0).mean() < 0.7


def test_many_chains_step_counts_model_unequal_speeds():
    w = wl.many_chains(m=4096, d=256, k=512, n_full=2000)
    assert w.k == 512 and 500 <= w.n_steps.min() and w.n_steps.max() <= 2000
    assert w.n_steps.max() > 1.5 * w.n_steps.min()


def test_wide_bf16_rows_are_bfloat16_bit_patterns():
    w = wl.wide_bf16(m=256, d=2048, k=8, n_levels=(80, 40, 20, 10))
    assert w.dense.dtype == np.uint16 and w.is_bf16 and w.row_bytes() == 4096
    assert w.n_steps.tolist() == [80, 80, 40, 40, 20, 20, 10, 10]
    back = wl.bf16_bits_to_f32(w.dense)
    assert abs(back.std() - 1 / np.sqrt(2048)) < 1e-3


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2.0 ** -8 + 2.0 ** -20, -3.0], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to the even mantissa (1.0);
    # 1 + 3*2^-8 ties between 1+2^-7 (odd) and 1+2^-6 (even): goes up
    got = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.0, 1.015625, 1.0078125, -3.0]


def test_sparse_hinge_structure():
    w = wl.sparse_hinge(m=20000, d=1 << 16, k=16, n_median=300)
    assert w.is_csr and w.row_ptr.shape == (20001,) and w.row_ptr[0] == 0
    lens = np.diff(w.row_ptr)
    assert lens.min() >= 1 and lens.max() <= 256 and 70 < lens.mean() < 90
    assert w.col_idx.dtype == np.int32 and w.col_idx.min() >= 0 and w.col_idx.max() < w.d
    starts = w.row_ptr[:-1]
    inc = np.diff(w.col_idx.astype(np.int64)) > 0
    inc[starts[1:] - 1] = True                       # row boundaries may go down
    assert inc.all()                                 # strictly ascending inside every row
    sq = np.add.reduceat(w.vals.astype(np.float64) ** 2, starts)
    np.testing.assert_allclose(sq, 1.0, rtol=1e-5)   # unit rows
    # Zipf head: a few low columns take a large share of all entries
    assert (w.col_idx < 64).mean() > 0.15
    assert set(np.unique(w.y)) == {-1.0, 1.0}
    again = wl.sparse_hinge(m=20000, d=1 << 16, k=16, n_median=300)
    assert np.array_equal(again.col_idx, w.col_idx) and np.array_equal(again.vals, w.vals)


def test_analog_binary_follows_the_papers_recipe():
    w = wl.analog_binary(m_train=3000, m_test=500, d=5000, n_fast=1000)
    assert w.is_csr and w.m == 3500 and w.meta["m_train"] == 3000
    lens = np.diff(w.row_ptr)
    assert lens.min() == 5 and lens.max() == 10
    assert w.n_steps.tolist() == [1000] * 8 + [200] * 2
    for r in (0, 1, 17, 3499):
        c = w.col_idx[w.row_ptr[r]:w.row_ptr[r + 1]].astype(np.int64)
        v = w.vals[w.row_ptr[r]:w.row_ptr[r + 1]]
        assert (np.diff(c) > 0).all() and c.max() < 5000
        np.testing.assert_allclose(v, 1 / np.sqrt(len(c)), rtol=1e-6)          # binary features, unit row
        score = sum(((i + 1) % 4) * (-1) ** (i + 1) for i in c.tolist())           # the paper's labelling rule
        assert w.y[r] == (1.0 if score > 0 else -1.0)
    assert 0.2 < (w.y > 0).mean() < 0.8


def test_delay_servers_rows_lie_close_to_one_direction():
    w = wl.delay_servers(m=1024, d=256, k=8, n_lo=30, n_hi=90, tau=3)
    assert w.dense.shape == (1024, 256) and w.dense.dtype == np.float32 and w.loss == wl.LOGISTIC
    assert w.meta["tau"] == 3 and w.meta["w_start"].dtype == np.float32 and w.meta["w_start"].shape == (256,)
    assert set(np.unique(w.y)) == {-1.0, 1.0} and 30 <= w.n_steps.min() and w.n_steps.max() <= 90
    # x_j = y_j * s_j * u + noise: the label-signed rows share one direction, lengths 0.6 .. 1, little across it
    X = w.dense.astype(np.float64) * w.y[:, None]
    u = X.mean(axis=0)
    u /= np.linalg.norm(u)
    along = X @ u
    across = np.linalg.norm(X - np.outer(along, u), axis=1)
    assert 0.59 < along.min() and along.max() < 1.01 and across.max() < 0.02
    # eta * (lambda + |x|^2) < 1 on every row, so the contraction rate of the Check function leaves an interval
    assert (w.eta * (w.lam + (w.dense.astype(np.float64) ** 2).sum(axis=1)) < 1).all()
    again = wl.delay_servers(m=1024, d=256, k=8, n_lo=30, n_hi=90, tau=3)
    assert np.array_equal(again.dense, w.dense) and np.array_equal(again.meta["w_start"], w.meta["w_start"])
    b = wl.delay_servers(m=64, d=64, k=2, n_lo=3, n_hi=5, bf16=True)
    assert b.dense.dtype == np.uint16 and b.is_bf16
