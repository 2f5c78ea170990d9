"""Pins of the CPU oracle against what the paper and the mathematics fix.

Each test names the passage it rests on.  None of the expected values comes
from the oracle itself or from the GPU path.
"""
import math

import numpy as np
import pytest
from scipy import optimize

from conftest import golden_rows
from oracle import oracle as orc


# ---------------------------------------------------------------- sample-index stream

@pytest.mark.parametrize("row", golden_rows("philox4x32_10_kat.txt"))
def test_philox_known_answers(row):
    """Published Philox4x32-10 known-answer vectors (Salmon et al., SC'11)."""
    words = [int(t, 16) for t in row.split()]
    got = orc.philox4x32_10(words[0:4], words[4:6])
    assert [int(v) for v in got] == words[6:10]


@pytest.mark.parametrize("row", golden_rows("sample_index_streams.txt"))
def test_index_streams_match_independent_values(row):
    head, tail = row.split(":")
    seed, chain, m, n0 = (int(t) for t in head.split())
    want = [int(t) for t in tail.split()]
    got = orc.sample_indices(seed, chain, n0, len(want), m)
    assert got.tolist() == want


def test_index_mapping_is_multiply_shift_of_word0():
    """index = floor(word0 * m / 2^32) with word0 from counter (step, chain), key = seed."""
    seed, chain, m = (5 << 32) | 77, 3, 1000003
    for step in (0, 1, 63, 64, (1 << 32) + 5):
        w0 = int(orc.philox4x32_10([step & 0xFFFFFFFF, step >> 32, chain, 0],
                                   [seed & 0xFFFFFFFF, seed >> 32])[0])
        assert orc.sample_indices(seed, chain, step, 1, m)[0] == (w0 * m) // (1 << 32)


def test_index_range_and_uniformity():
    m = 10
    idx = orc.sample_indices(123, 0, 0, 200000, m)
    assert idx.min() >= 0 and idx.max() < m
    counts = np.bincount(idx, minlength=m)
    chi2 = ((counts - 20000.0) ** 2 / 20000.0).sum()
    assert chi2 < 40.0          # 9 degrees of freedom; 40 is far in the tail
    assert (orc.sample_indices(9, 4, 0, 100, 1) == 0).all()
    big = orc.sample_indices(9, 4, 0, 1000, (1 << 32) - 1)
    assert big.max() < (1 << 32) - 1 and big.max() > (1 << 31)


def test_index_stream_from_an_offset_is_a_slice_of_the_stream():
    whole = orc.sample_indices(9, 3, 0, 300, 1000)
    for n0 in (0, 1, 63, 64, 65, 250):
        assert np.array_equal(orc.sample_indices(9, 3, n0, 40, 1000), whole[n0:n0 + 40])


# ------------------------------------------------ partition-and-shuffle sampling (Algorithm 1 as written)

@pytest.mark.parametrize("m,k", [(1, 1), (2, 1), (2, 2), (3, 2), (5, 5), (16, 3), (17, 4), (64, 64), (1000, 7),
                                 (4097, 10), (65536, 9), (65537, 8)])
def test_shards_partition_the_rows_and_every_node_sees_its_share_once(m, k):
    """"Randomly partition the examples ... randomly shuffle the data on each node": over its
    first m_i steps a node sees m_i different rows, the nodes' rows are disjoint, together they
    are every row, and the share sizes differ by at most one."""
    seen = []
    for i in range(k):
        own = (i + 1) * m // k - i * m // k
        assert own >= 1 and abs(own - m / k) < 1
        rows = orc.shard_indices(12345, i, k, 0, own, m)
        assert rows.min() >= 0 and rows.max() < m and np.unique(rows).size == own
        again = orc.shard_indices(12345, i, k, own, min(own, 50), m)      # a second pass repeats the order
        assert np.array_equal(again, rows[:again.size])
        assert np.array_equal(orc.shard_indices(12345, i, k, 3, 5, m), np.resize(rows, 8)[3:8])
        seen.append(rows)
    allrows = np.concatenate(seen)
    assert np.array_equal(np.sort(allrows), np.arange(m))


def test_shard_order_is_shuffled_and_depends_on_the_seed():
    m, k = 10007, 4
    a = orc.shard_indices(1, 0, k, 0, 2000, m)
    b = orc.shard_indices(2, 0, k, 0, 2000, m)
    assert not np.array_equal(a, b)
    # not the identity, not sorted, and spread over the whole range: the mean rank of a node's rows is m/2
    assert (np.diff(a) > 0).mean() == pytest.approx(0.5, abs=0.05)
    assert a.mean() == pytest.approx(m / 2, rel=0.05) and b.mean() == pytest.approx(m / 2, rel=0.05)
    # which node a row lands on is balanced over seeds: row 0 visits every node
    owners = set()
    for seed in range(40):
        for i in range(k):
            if 0 in orc.shard_indices(seed, i, k, 0, (i + 1) * m // k - i * m // k, m):
                owners.add(i)
    assert owners == set(range(k))


def test_shard_sampling_rejects_bad_arguments():
    for args in [(0, 0, 3, 0, 1, 2), (0, 3, 3, 0, 1, 10), (0, -1, 3, 0, 1, 10), (0, 0, 0, 0, 1, 10), (0, 0, 1, 0, 1, 0)]:
        with pytest.raises(ValueError):
            orc.shard_indices(*args)


def test_index_streams_differ_by_chain_step_and_seed():
    a = orc.sample_indices(0, 0, 0, 64, 1 << 20)
    assert not np.array_equal(a, orc.sample_indices(0, 1, 0, 64, 1 << 20))
    assert not np.array_equal(a, orc.sample_indices(1, 0, 0, 64, 1 << 20))
    assert np.array_equal(a[10:], orc.sample_indices(0, 0, 10, 54, 1 << 20))


# ---------------------------------------------------------------- weights (Eq. 6, Eq. 8)

@pytest.mark.parametrize("row", golden_rows("weights_cases.txt"))
def test_weights_hand_and_decimal_cases(row):
    rate_s, n_s, a_s = row.split(";")
    n = [int(t) for t in n_s.split()]
    want = np.array([float(t) for t in a_s.split()])
    got = orc.weights_rate(n, float(rate_s))
    # the rate itself is only known to half an ulp as a double; a power T magnifies that T times
    rtol = 1e-13 + (max(n) - min(n)) * 2.3e-16
    np.testing.assert_allclose(got, want, rtol=rtol, atol=0)


def test_weights_eq6_uses_one_minus_eta_lambda():
    got = orc.weights([3, 1], 0.5, 0.5)
    np.testing.assert_allclose(got, [16 / 25, 9 / 25], rtol=1e-15)
    got = orc.weights([4, 2, 1], 0.5, 1.0)
    np.testing.assert_allclose(got, [8 / 11, 2 / 11, 1 / 11], rtol=1e-15)


def test_equal_step_counts_give_uniform_average():
    """All delays zero: Eq. 6 turns into the 1/k of SimuParallel SGD (Algorithm 2)."""
    for k in (1, 2, 7, 64):
        a = orc.weights([1234] * k, 0.05, 1e-4)
        assert np.array_equal(a, np.full(k, 1.0 / k))


def test_weight_laws():
    rng = np.random.default_rng(0)
    n = rng.integers(0, 50000, size=33)
    eta, lam = 0.1, 1e-4
    a = orc.weights(n, eta, lam)
    assert abs(a.sum() - 1.0) < 1e-14                       # premise of Lemma 2
    rho = 1.0 - eta * lam
    i, j = 3, 17
    assert a[i] / a[j] == pytest.approx(rho ** float(n[j] - n[i]), rel=1e-12)
    order = np.argsort(n)
    assert (np.diff(a[order]) >= 0).all()                   # more delay, less weight
    a0 = orc.weights(n, eta, 0.0)                           # lambda = 0: rate 1, uniform
    np.testing.assert_allclose(a0, 1.0 / n.size, rtol=1e-15)


def test_weights_idle_nodes():
    """Nodes that did no work keep the weight of a delay of t steps (Fig. 7 set-up)."""
    a = orc.weights([100, 100, 0, 0], 0.5, 0.02)            # rate 0.99
    r = 0.99 ** 100
    np.testing.assert_allclose(a, np.array([1, 1, r, r]) / (2 + 2 * r), rtol=1e-13)
    assert np.array_equal(orc.weights([0, 0, 0], 0.5, 0.02), np.full(3, 1 / 3))


def test_weights_reject_bad_arguments():
    for bad in [dict(n=[1, -1], eta=0.1, lam=0.1), dict(n=[1], eta=0.0, lam=0.1),
                dict(n=[1], eta=2.0, lam=0.5), dict(n=[1], eta=0.1, lam=-1.0)]:
        with pytest.raises(ValueError):
            orc.weights(bad["n"], bad["eta"], bad["lam"])


def test_benefit_condition():
    """2 sum rate^T_i > sqrt(k) + k (Eq. 7): true for the tiny workload, false for n={3,1}."""
    rho = 1 - 1e-5
    lhs = 2 * sum(rho ** t for t in (0, 200, 400, 600))
    assert orc.benefit_margin([1000, 800, 600, 400], rho) == pytest.approx(lhs - 6.0, rel=1e-12)
    assert lhs - 6.0 == pytest.approx(1.97605578468828733, rel=1e-12)     # decimal arithmetic
    assert orc.benefit_margin([3, 1], 0.75) == pytest.approx(3.125 - (math.sqrt(2) + 2), rel=1e-13)
    assert orc.benefit_margin([3, 1], 0.75) < 0 < orc.benefit_margin([5, 5, 5], 0.9)


# ---------------------------------------------------------------- combine (Algorithm 1, last line)

def test_combine_linearity_selection_and_mean():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((5, 37))
    for i in range(5):
        e = np.zeros(5)
        e[i] = 1.0
        assert np.array_equal(orc.combine(W, e), W[i])
    np.testing.assert_allclose(orc.combine(W, np.full(5, 0.2)), W.mean(axis=0), rtol=1e-14, atol=1e-16)
    a, b = rng.random(5), rng.random(5)
    np.testing.assert_allclose(orc.combine(W, 2 * a - 3 * b),
                               2 * orc.combine(W, a) - 3 * orc.combine(W, b), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(orc.combine(W, a), a @ W, rtol=1e-13, atol=1e-15)   # library GEMV


# ---------------------------------------------------------------- the SGD step (Eq. 4, Eq. 5)

def _hand_matrix(dtype=np.float32):
    X = np.array([[1, 0], [0, 2], [1, 1]], dtype=dtype)
    y = np.array([1, -1, 1], dtype=np.float32)
    return X, y


def test_hinge_hand_case_all_prefixes():
    X, y = _hand_matrix()
    order = [0, 1, 2, 0, 2, 0]
    for row in golden_rows("hinge_hand_case.txt"):
        steps, w0, w1 = row.split()
        w, _ = orc.sgd(orc.Dense(X), y, order[: int(steps)], 0.5, 0.5, orc.HINGE)
        assert w.tolist() == [float(w0), float(w1)]          # exact binary fractions
    _, closest = orc.sgd(orc.Dense(X), y, order, 0.5, 0.5, orc.HINGE)
    assert closest == 0.1015625


def test_hinge_hand_case_csr_f64_and_bf16_storage():
    X, y = _hand_matrix()
    order = [0, 1, 2, 0, 2, 0]
    want = [0.98583984375, 0.26953125]
    csr = orc.CSR([0, 1, 2, 4], [0, 1, 0, 1], [1, 2, 1, 1], 2)
    for mode in (orc.PLAIN, orc.LAZY):
        w, mm = orc.sgd(csr, y, order, 0.5, 0.5, orc.HINGE, csr_mode=mode)
        np.testing.assert_allclose(w, want, rtol=1e-15)
        assert mm == pytest.approx(0.1015625, rel=1e-14)
    w, _ = orc.sgd(orc.Dense(X.astype(np.float64)), y, order, 0.5, 0.5, orc.HINGE)
    assert w.tolist() == want
    bits = (X.view(np.uint32) >> 16).astype(np.uint16)        # these values are exact in bfloat16
    w, _ = orc.sgd(orc.Dense(bits), y, order, 0.5, 0.5, orc.HINGE)
    assert w.tolist() == want


@pytest.mark.parametrize("loss,factor", [(orc.HINGE, 1.0), (orc.LOGISTIC, 0.5)])
def test_first_step_from_zero_is_closed_form(loss, factor):
    """From w_0 = 0: yhat = 0, so hinge fires (0 < 1) and the logistic slope is -y/2."""
    rng = np.random.default_rng(2)
    X = rng.standard_normal((6, 9)).astype(np.float32)
    y = np.array([1, -1, 1, -1, -1, 1], dtype=np.float32)
    eta, lam = 0.3, 0.2
    for j in range(6):
        w, _ = orc.sgd(orc.Dense(X), y, [j], eta, lam, loss)
        np.testing.assert_allclose(w, factor * eta * float(y[j]) * X[j].astype(np.float64), rtol=1e-15)


def test_hinge_same_row_geometric_series_then_pure_decay():
    """One row visited over and over: while y*yhat < 1 every step adds eta*y*x to the shrunk
    vector, w_n = eta*y*x*(1 - rho^n)/(1 - rho); once y*yhat >= 1 only the shrink acts."""
    x = np.array([[0.5, -0.25, 0.125]], dtype=np.float32)
    y = np.array([-1.0], dtype=np.float32)
    eta, lam = 0.0625, 0.5
    rho = 1 - eta * lam
    sq = float((x.astype(np.float64) ** 2).sum())
    n = 12
    assert eta * sq * (1 - rho ** (n - 1)) / (1 - rho) < 1       # still active at step n
    w, _ = orc.sgd(orc.Dense(x), y, [0] * n, eta, lam, orc.HINGE)
    np.testing.assert_allclose(w, eta * -1.0 * x[0].astype(np.float64) * (1 - rho ** n) / (1 - rho), rtol=1e-14)
    # large first step: margin 4 after one update, so the next steps only decay
    xb = np.array([[2.0, 0.0, 0.0]], dtype=np.float32)
    w, _ = orc.sgd(orc.Dense(xb), np.array([1.0], dtype=np.float32), [0] * 5, 1.0, 0.25, orc.HINGE)
    np.testing.assert_allclose(w, [2.0 * 0.75 ** 4, 0, 0], rtol=1e-15)


def _objective(loss, lam, w, x, y):
    """c^i(w) = lambda/2 |w|^2 + L(x, y, w.x)  -- Eq. 4, written as a value, not a gradient."""
    z = y * float(w @ x)
    L = max(0.0, 1.0 - z) if loss == orc.HINGE else math.log1p(math.exp(-z))
    return 0.5 * lam * float(w @ w) + L


@pytest.mark.parametrize("loss", [orc.HINGE, orc.LOGISTIC])
@pytest.mark.parametrize("storage", ["dense", "csr_plain", "csr_lazy"])
def test_step_is_minus_eta_times_numerical_gradient(loss, storage):
    """(w_{n-1} - w_n)/eta must equal the gradient of Eq. 4 at w_{n-1} (Eq. 5); the gradient
    is taken here by central differences of the objective value."""
    rng = np.random.default_rng(3)
    d = 7
    Xd = rng.standard_normal((4, d)).astype(np.float32)
    Xd[rng.random((4, d)) < 0.4] = 0
    Xd[:, 0] = 1.0
    y = np.array([1, -1, -1, 1], dtype=np.float32)
    if storage == "dense":
        X, mode = orc.Dense(Xd), orc.PLAIN
    else:
        rp, ci, va = [0], [], []
        for r in range(4):
            nz = np.nonzero(Xd[r])[0]
            ci += nz.tolist()
            va += Xd[r, nz].tolist()
            rp.append(len(ci))
        X, mode = orc.CSR(rp, ci, va, d), (orc.PLAIN if storage == "csr_plain" else orc.LAZY)
    eta, lam = 0.05, 0.3
    for trial in range(8):
        w0 = rng.standard_normal(d) * 0.7
        j = trial % 4
        x = Xd[j].astype(np.float64)
        if loss == orc.HINGE and abs(1 - float(y[j]) * float(w0 @ x)) < 1e-3:
            continue
        w1, _ = orc.sgd(X, y, [j], eta, lam, loss, w0=w0, csr_mode=mode)
        h = 1e-6
        grad = np.array([(_objective(loss, lam, w0 + h * e, x, float(y[j])) -
                          _objective(loss, lam, w0 - h * e, x, float(y[j]))) / (2 * h)
                         for e in np.eye(d)])
        np.testing.assert_allclose((w0 - w1) / eta, grad, rtol=1e-6, atol=1e-8)


def test_logistic_single_row_converges_to_stationary_point():
    """On a one-row data set SGD is gradient descent on c; its limit solves
    lambda*w = y*x / (1 + exp(y*w.x)).  The root is found with a library solver."""
    x = np.array([[1.5, -0.5]], dtype=np.float32)
    y = np.array([1.0], dtype=np.float32)
    eta, lam = 0.2, 0.1
    w, _ = orc.sgd(orc.Dense(x), y, [0] * 4000, eta, lam, orc.LOGISTIC)
    sq = 2.5
    # w = alpha * x with lam*alpha = 1/(1+exp(alpha*|x|^2))
    alpha = optimize.brentq(lambda a: lam * a - 1.0 / (1.0 + math.exp(a * sq)), 0.0, 10.0, xtol=1e-15)
    np.testing.assert_allclose(w, alpha * x[0].astype(np.float64), rtol=1e-10)
    res = optimize.minimize(lambda v: _objective(orc.LOGISTIC, lam, v, x[0].astype(np.float64), 1.0),
                            np.zeros(2), method="BFGS", options={"gtol": 1e-10})
    np.testing.assert_allclose(w, res.x, rtol=1e-5)


def test_logistic_chain_contracts_at_rate_one_minus_eta_lambda():
    """Two chains fed the same rows from different starts approach each other at least as
    fast as (1 - eta*lambda)^n for a small enough step (Theorem 3; section IV, Lemma 4 remark)."""
    rng = np.random.default_rng(4)
    X = (rng.standard_normal((50, 6)) / 3).astype(np.float32)
    y = np.where(rng.random(50) < 0.5, 1.0, -1.0).astype(np.float32)
    idx = rng.integers(0, 50, size=300)
    eta, lam = 0.1, 0.05
    rho = 1 - eta * lam
    a0, b0 = rng.standard_normal(6), rng.standard_normal(6)
    prev = np.linalg.norm(a0 - b0)
    for n in (1, 2, 10, 100, 300):
        wa, _ = orc.sgd(orc.Dense(X), y, idx[:n], eta, lam, orc.LOGISTIC, w0=a0)
        wb, _ = orc.sgd(orc.Dense(X), y, idx[:n], eta, lam, orc.LOGISTIC, w0=b0)
        dist = np.linalg.norm(wa - wb)
        assert dist <= prev * rho ** n * (1 + 1e-12)
    # with y*yhat >= 1 everywhere hinge has no gradient: the distance shrinks by exactly rho^n
    Xh = np.array([[3.0, 0.0]], dtype=np.float32)
    yh = np.array([1.0], dtype=np.float32)
    wa, _ = orc.sgd(orc.Dense(Xh), yh, [0] * 7, eta, lam, orc.HINGE, w0=[1.0, 2.0])
    wb, _ = orc.sgd(orc.Dense(Xh), yh, [0] * 7, eta, lam, orc.HINGE, w0=[2.0, -1.0])
    np.testing.assert_allclose(wa - wb, rho ** 7 * np.array([-1.0, 3.0]), rtol=1e-14)


def _brute_force_chain(X, y, idx, eta, lam, loss):
    """Tiny-input brute force with Python floats, one coordinate at a time."""
    d = X.shape[1]
    w = [0.0] * d
    for j in idx:
        x = [float(v) for v in X[j]]
        yhat = math.fsum(w[c] * x[c] for c in range(d))
        yy = float(y[j])
        if loss == orc.HINGE:
            slope = -yy if yy * yhat < 1.0 else 0.0
        else:
            slope = -yy / (1.0 + math.exp(yy * yhat))
        w = [w[c] - eta * (lam * w[c] + slope * x[c]) for c in range(d)]   # Eq. 5 as printed
    return np.array(w)


@pytest.mark.parametrize("loss", [orc.HINGE, orc.LOGISTIC])
def test_chain_against_brute_force(loss):
    rng = np.random.default_rng(5)
    X = rng.standard_normal((40, 12)).astype(np.float32)
    y = np.where(rng.random(40) < 0.5, 1.0, -1.0).astype(np.float32)
    idx = orc.sample_indices(11, 2, 0, 400, 40)
    w, _ = orc.sgd(orc.Dense(X), y, idx, 0.05, 0.01, loss)
    np.testing.assert_allclose(w, _brute_force_chain(X, y, idx, 0.05, 0.01, loss), rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- storage variants agree

def _random_csr(rng, m, d, nnz):
    rp, ci, va = [0], [], []
    for _ in range(m):
        c = np.sort(rng.choice(d, size=rng.integers(1, nnz + 1), replace=False))
        ci += c.tolist()
        va += rng.standard_normal(c.size).tolist()
        rp.append(len(ci))
    return orc.CSR(rp, ci, va, d)


@pytest.mark.parametrize("loss", [orc.HINGE, orc.LOGISTIC])
def test_csr_equals_dense_and_lazy_equals_plain(loss):
    rng = np.random.default_rng(6)
    csr = _random_csr(rng, 30, 25, 6)
    dense = np.zeros((30, 25), dtype=np.float32)
    for r in range(30):
        lo, hi = csr.row_ptr[r], csr.row_ptr[r + 1]
        dense[r, csr.col_idx[lo:hi]] = csr.vals[lo:hi]
    y = np.where(rng.random(30) < 0.5, 1.0, -1.0).astype(np.float32)
    idx = rng.integers(0, 30, size=500)
    wd, md = orc.sgd(orc.Dense(dense), y, idx, 0.1, 0.02, loss)
    wp, mp = orc.sgd(csr, y, idx, 0.1, 0.02, loss, csr_mode=orc.PLAIN)
    wl, ml = orc.sgd(csr, y, idx, 0.1, 0.02, loss, csr_mode=orc.LAZY)
    np.testing.assert_allclose(wp, wd, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(wl, wp, rtol=1e-12, atol=1e-14)
    assert md == pytest.approx(mp, rel=1e-9) and ml == pytest.approx(mp, rel=1e-9)


def test_lazy_scale_survives_heavy_shrink():
    rng = np.random.default_rng(7)
    csr = _random_csr(rng, 10, 8, 3)
    y = np.ones(10, dtype=np.float32)
    idx = rng.integers(0, 10, size=3000)
    wp, _ = orc.sgd(csr, y, idx, 0.5, 0.9, orc.LOGISTIC, csr_mode=orc.PLAIN)   # rho^n ~ 1e-780
    wl, _ = orc.sgd(csr, y, idx, 0.5, 0.9, orc.LOGISTIC, csr_mode=orc.LAZY)
    assert np.isfinite(wl).all() and np.abs(wp).max() > 1e-3
    np.testing.assert_allclose(wl, wp, rtol=1e-11, atol=1e-14)


def test_bf16_rows_are_widened_exactly():
    rng = np.random.default_rng(8)
    Xf = rng.standard_normal((20, 16)).astype(np.float32)
    bits = (Xf.view(np.uint32) >> 16).astype(np.uint16)                # truncation is fine here
    widened = (bits.astype(np.uint32) << 16).view(np.float32)
    y = np.where(rng.random(20) < 0.5, 1.0, -1.0).astype(np.float32)
    idx = rng.integers(0, 20, size=200)
    wb, _ = orc.sgd(orc.Dense(bits), y, idx, 0.05, 0.01, orc.LOGISTIC)
    wf, _ = orc.sgd(orc.Dense(widened), y, idx, 0.05, 0.01, orc.LOGISTIC)
    assert np.array_equal(wb, wf)


# ---------------------------------------------------------------- whole path (Algorithm 1)

def _small_problem(seed=9, m=64, d=10):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((m, d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    return orc.Dense(X), y


def test_single_chain_is_sequential_sgd():
    """k = 1: weight 1, the output is the one chain's last iterate."""
    X, y = _small_problem()
    v, W, a = orc.wpsgd(X, y, [250], 0.05, 0.01, orc.HINGE, seed=3)
    idx = orc.sample_indices(3, 0, 0, 250, X.m)
    w, _ = orc.sgd(X, y, idx, 0.05, 0.01, orc.HINGE)
    assert a.tolist() == [1.0] and np.array_equal(v, w) and np.array_equal(W[0], w)


def test_equal_lengths_reduce_to_plain_model_average():
    X, y = _small_problem()
    v, W, a = orc.wpsgd(X, y, [120] * 6, 0.05, 0.01, orc.LOGISTIC, seed=1)
    np.testing.assert_allclose(v, W.mean(axis=0), rtol=1e-13, atol=1e-16)
    assert not np.allclose(W[0], W[1])          # chains do see different rows


def test_chain_rows_follow_their_own_streams_and_subsets():
    X, y = _small_problem()
    n = [90, 0, 45, 200]
    W, mm = orc.run_chains(X, y, n, 0.05, 0.01, orc.HINGE, seed=5)
    for i, steps in enumerate(n):
        w, m_i = orc.sgd(X, y, orc.sample_indices(5, i, 0, steps, X.m), 0.05, 0.01, orc.HINGE)
        assert np.array_equal(W[i], w)
        assert mm[i] == m_i
    assert (W[1] == 0).all() and math.isinf(mm[1])          # idle chain: w stays w_0 = 0
    Wsub, _ = orc.run_chains(X, y, n, 0.05, 0.01, orc.HINGE, seed=5, chain_ids=[3, 0], threads=1)
    assert np.array_equal(Wsub[0], W[3]) and np.array_equal(Wsub[1], W[0])


@pytest.mark.parametrize("loss", [orc.HINGE, orc.LOGISTIC])
def test_constant_start_value_of_the_experiments(loss):
    """Section V starts every node from a constant vector (4 there) instead of Algorithm 1's zero.
    With w_0 = c*1 the first step is closed-form (Eq. 5 with Eq. 4): yhat = c*sum(x_j) and
    w_1 = (1 - eta*lambda)*c*1 - eta*g*x_j; a chain of no steps returns c*1; longer chains are the
    sequential recursion started from c*1."""
    X, y = _small_problem()
    eta, lam, c = 0.05, 0.01, 4.0
    n = [1, 0, 37, 150]
    W, mm = orc.run_chains(X, y, n, eta, lam, loss, seed=11, w0_fill=c)
    j = int(orc.sample_indices(11, 0, 0, 1, X.m)[0])
    x = X.data[j].astype(np.float64)
    yj = float(y[j])
    yhat = c * x.sum()
    g = (-yj if yj * yhat < 1.0 else 0.0) if loss == orc.HINGE else -yj / (1.0 + math.exp(yj * yhat))
    np.testing.assert_allclose(W[0], (1.0 - eta * lam) * c - eta * g * x, rtol=1e-14, atol=1e-15)
    assert (W[1] == c).all() and math.isinf(mm[1])
    for i in (2, 3):
        w, m_i = orc.sgd(X, y, orc.sample_indices(11, i, 0, n[i], X.m), eta, lam, loss, w0=np.full(X.d, c))
        assert np.array_equal(W[i], w) and mm[i] == m_i
    # the start value matters: the same chains from zero end elsewhere
    W0, _ = orc.run_chains(X, y, n, eta, lam, loss, seed=11)
    assert not np.allclose(W0[3], W[3])
    # a sparse copy of the matrix, both update modes
    rp = np.arange(0, X.m * X.d + 1, X.d, dtype=np.int64)
    ci = np.tile(np.arange(X.d, dtype=np.int32), X.m)
    Xs = orc.CSR(rp, ci, X.data.reshape(-1), X.d)
    for mode in (orc.PLAIN, orc.LAZY):
        Ws, _ = orc.run_chains(Xs, y, n, eta, lam, loss, seed=11, w0_fill=c, csr_mode=mode)
        np.testing.assert_allclose(Ws, W, rtol=1e-12, atol=1e-14)


def test_weighted_output_is_the_weighted_sum_of_chain_outputs():
    X, y = _small_problem()
    n = [300, 100, 200]
    v, W, a = orc.wpsgd(X, y, n, 0.5, 0.1, orc.HINGE, seed=2)       # rate 0.95: visibly unequal
    rho = 0.95
    raw = np.array([1.0, rho ** 200, rho ** 100])
    np.testing.assert_allclose(a, raw / raw.sum(), rtol=1e-13)
    np.testing.assert_allclose(v, (raw / raw.sum()) @ W, rtol=1e-13, atol=1e-16)


# ---------------------------------------------------------------- periodic averaging (Section III, Deduction 2)

def test_one_chain_averaged_with_itself_is_one_long_chain():
    """k = 1: the average of one model is that model, so S spans of n steps are S*n sequential
    steps of the chain's own stream (pins the restart vector and the stream offsets)."""
    X, y = _small_problem()
    for loss in (orc.HINGE, orc.LOGISTIC):
        v = orc.run_spans(X, y, [70], 4, 0.05, 0.01, loss, seed=3)
        w, _ = orc.sgd(X, y, orc.sample_indices(3, 0, 0, 280, X.m), 0.05, 0.01, loss)
        assert np.array_equal(v, w)
    start = np.linspace(-1.0, 1.0, X.d)
    v = orc.run_spans(X, y, [70], 2, 0.05, 0.01, orc.HINGE, seed=3, w0=start)
    w, _ = orc.sgd(X, y, orc.sample_indices(3, 0, 0, 140, X.m), 0.05, 0.01, orc.HINGE, w0=start)
    assert np.array_equal(v, w)
    v = orc.run_spans(X, y, [40], 3, 0.05, 0.01, orc.HINGE, seed=3, shards=True)
    w, _ = orc.sgd(X, y, orc.shard_indices(3, 0, 1, 0, 120, X.m), 0.05, 0.01, orc.HINGE)
    assert np.array_equal(v, w)


def test_one_span_is_algorithm_1_and_equal_chains_take_the_plain_mean_every_span():
    X, y = _small_problem()
    n = [90, 30, 60]
    v1, _, _ = orc.wpsgd(X, y, n, 0.5, 0.1, orc.HINGE, seed=2)
    assert np.array_equal(orc.run_spans(X, y, n, 1, 0.5, 0.1, orc.HINGE, seed=2), v1)
    # second span by hand: every chain restarts from v1 at its own offset, weights as in Eq. 6
    rho = 0.95
    raw = np.array([1.0, rho ** 60, rho ** 30])
    W2 = np.stack([orc.sgd(X, y, orc.sample_indices(2, i, n[i], n[i], X.m), 0.5, 0.1, orc.HINGE, w0=v1)[0]
                   for i in range(3)])
    np.testing.assert_allclose(orc.run_spans(X, y, n, 2, 0.5, 0.1, orc.HINGE, seed=2),
                               (raw / raw.sum()) @ W2, rtol=1e-12, atol=1e-15)
    # equal chains: the plain mean after each span (the averaging of Deduction 1)
    v = np.zeros(X.d)
    for s in range(3):
        v = np.mean([orc.sgd(X, y, orc.sample_indices(7, i, 50 * s, 50, X.m), 0.05, 0.01, orc.LOGISTIC, w0=v)[0]
                     for i in range(4)], axis=0)
    np.testing.assert_allclose(orc.run_spans(X, y, [50] * 4, 3, 0.05, 0.01, orc.LOGISTIC, seed=7), v,
                               rtol=1e-12, atol=1e-15)


def test_span_validity_condition():
    """k / sum_j rho^{T_j} * rho^{span} (below Deduction 2): rho^span for equal chains, k times
    the fastest chain's Eq. 6 weight times rho^span in general, 1 without regularisation."""
    assert orc.span_condition([50, 50, 50], 0.99) == pytest.approx(0.99 ** 50, rel=1e-14)
    assert orc.span_condition([100, 0], 0.999) == pytest.approx(2.0 / (1.0 + 0.999 ** 100) * 0.999 ** 100, rel=1e-14)
    n = [100, 80, 60, 100]
    a = orc.weights_rate(n, 0.999)
    assert orc.span_condition(n, 0.999) == pytest.approx(4 * a[0] * 0.999 ** 100, rel=1e-13)
    assert orc.span_condition([7, 3, 5], 1.0) == 1.0
    # With T_j = span - D_j the expression equals k / sum_j rho^{-D_j}: the harmonic-mean form shows
    # that it never exceeds 1 and reaches 1 only when no chain moves.
    for n, rate in (([10, 3, 0, 7], 0.97), ([1, 1], 0.5), ([0, 0, 5], 0.999)):
        assert orc.span_condition(n, rate) == pytest.approx(len(n) / sum(rate ** -d for d in n), rel=1e-13)
        assert orc.span_condition(n, rate) < 1.0
    assert orc.span_condition([0, 0, 0], 0.9) == 1.0
    with pytest.raises(Exception):
        orc.span_condition([3, -1], 0.9)
    with pytest.raises(Exception):
        orc.span_condition([3, 1], 1.5)


# ---------------------------------------------------------------- objective (Eq. 3, Eq. 4)

def test_objective_closed_forms():
    X, y = _hand_matrix()
    zero = np.zeros(2)
    obj, err = orc.objective(orc.Dense(X), y, zero, 0.3, orc.HINGE)
    assert obj == 1.0 and err == 1.0
    obj, _ = orc.objective(orc.Dense(X), y, zero, 0.3, orc.LOGISTIC)
    assert obj == pytest.approx(math.log(2.0), rel=1e-15)
    w = np.array([2.0, 1.0])     # margins y*w.x: 2, -2, 3 -> hinge 0, 3, 0 ; errors 1 of 3
    obj, err = orc.objective(orc.Dense(X), y, w, 0.5, orc.HINGE)
    assert obj == pytest.approx(0.25 * 5.0 + 1.0, rel=1e-15) and err == pytest.approx(1 / 3)
    csr = orc.CSR([0, 1, 2, 4], [0, 1, 0, 1], [1, 2, 1, 1], 2)
    assert orc.objective(csr, y, w, 0.5, orc.HINGE) == (obj, err)
    obj, _ = orc.objective(csr, y, w, 0.0, orc.LOGISTIC)
    want = (math.log1p(math.exp(-2)) + math.log1p(math.exp(2)) + math.log1p(math.exp(-3))) / 3
    assert obj == pytest.approx(want, rel=1e-14)


def test_hinge_takes_zero_slope_exactly_at_the_kink():
    """The paper names hinge loss without choosing a subgradient at y*yhat == 1; the implementation
    takes 0 there (the step fires only on strict inequality)."""
    X = np.array([[1.0, 0.0]], dtype=np.float32)
    y = np.array([1.0], dtype=np.float32)
    w, closest = orc.sgd(orc.Dense(X), y, [0, 0, 0], 1.0, 0.0, orc.HINGE)
    assert w.tolist() == [1.0, 0.0] and closest == 0.0


# ---------------------------------------------------------------- delay SGD with the Check function
# (Section IV, Algorithms 3 and 4; the proof of Lemma 4 in the appendix)

def _aligned_rows(rng, m, d, noise):
    """Rows that nearly share one direction, so that projections on successive samples move the same
    way and the Check function accepts more than the first update."""
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    X = np.outer(0.6 + 0.4 * rng.random(m), u) + noise * rng.standard_normal((m, d))
    return X.astype(np.float32), np.ones(m, dtype=np.float32)


@pytest.mark.parametrize("loss", [orc.HINGE, orc.LOGISTIC])
def test_delay_zero_without_check_is_the_plain_chain(loss):
    """With no delay the server's update is Eq. 5 on the newest iterate."""
    rng = np.random.default_rng(21)
    X = rng.standard_normal((50, 13)).astype(np.float32)
    y = np.where(rng.random(50) < 0.5, 1.0, -1.0).astype(np.float32)
    idx = orc.sample_indices(3, 1, 0, 300, 50)
    w0 = rng.standard_normal(13)
    want, _ = orc.sgd(orc.Dense(X), y, idx, 0.05, 0.02, loss, w0=w0)
    got, accepted, _ = orc.delay_sgd(orc.Dense(X), y, idx, 0.05, 0.02, loss, 0, w0=w0, check=False)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)
    assert accepted == 300


def test_the_first_updates_of_a_delayed_server_all_see_the_start_vector():
    """Until tau + 1 updates are done the gradient is evaluated at w_0 = 0, where the hinge slope is
    -y and the regulariser vanishes: w_n = eta * sum of y_j x_j over the samples so far."""
    rng = np.random.default_rng(22)
    X = rng.standard_normal((20, 7)).astype(np.float32)
    y = np.where(rng.random(20) < 0.5, 1.0, -1.0).astype(np.float32)
    tau, eta = 5, 0.125
    idx = [3, 17, 3, 8, 0, 11, 19]
    for n in range(1, tau + 2):
        w, accepted, _ = orc.delay_sgd(orc.Dense(X), y, idx[:n], eta, 0.3, orc.HINGE, tau, check=False)
        want = eta * sum(float(y[j]) * X[j].astype(np.float64) for j in idx[:n])
        np.testing.assert_allclose(w, want, rtol=1e-14, atol=1e-16)
        assert accepted == n


@pytest.mark.parametrize("loss", [orc.HINGE, orc.LOGISTIC])
@pytest.mark.parametrize("tau", [1, 3])
def test_one_row_over_and_over_follows_the_scalar_recurrences_in_the_proof_of_lemma_4(loss, tau):
    """Proof of Lemma 4: along the sample, alpha_{n+1} = alpha_n - eta*lambda*alpha_{n-tau}
    - eta*u(alpha_{n-tau})*beta^2; across it, the perpendicular part obeys
    p_{n+1} = p_n - eta*lambda*p_{n-tau}.  The iterate is alpha*x/beta^2 + p."""
    x = np.array([[0.5, -1.0, 0.25, 2.0]], dtype=np.float32)
    yy = -1.0
    xd = x[0].astype(np.float64)
    beta2 = float(xd @ xd)
    w0 = np.array([0.3, 0.1, -0.7, 0.2])
    eta, lam, n = 0.03, 0.4, 40
    alpha = [float(w0 @ xd)]
    perp = [w0 - alpha[0] / beta2 * xd]
    for t in range(n):
        a_old, p_old = alpha[max(t - tau, 0)], perp[max(t - tau, 0)]
        u = (-yy if yy * a_old < 1.0 else 0.0) if loss == orc.HINGE else -yy / (1.0 + math.exp(yy * a_old))
        alpha.append(alpha[t] - eta * lam * a_old - eta * u * beta2)
        perp.append(perp[t] - eta * lam * p_old)
    w, accepted, _ = orc.delay_sgd(orc.Dense(x), np.array([yy], dtype=np.float32), [0] * n, eta, lam, loss, tau,
                                   w0=w0, check=False)
    np.testing.assert_allclose(w, alpha[n] / beta2 * xd + perp[n], rtol=1e-12, atol=1e-14)
    assert accepted == n


def test_check_function_on_hand_triples():
    """Algorithm 4 on numbers worked by hand.  Length_min = (L_b - rate*L_a)/(1 - rate) is the point v
    with (L_b - v)/(L_a - v) = rate; the new projection has to lie between L_b and it."""
    # rising: L_a = 0, L_b = 1, rate 1/2 -> Length_min = 2, interval [1, 2]
    for Lc, want in ((1.5, True), (1.0, True), (2.0, True), (2.5, False), (0.5, False)):
        assert orc.check_triple(0.0, 1.0, Lc, 4.0, 3.0, 0.5)[0] is want
    # falling: L_a = 4, L_b = 3, rate 1/2 -> Length_min = (3 - 2)/(1/2) = 2, interval [2, 3]
    for Lc, want in ((2.5, True), (2.0, True), (3.0, True), (1.875, False), (3.25, False)):
        assert orc.check_triple(4.0, 3.0, Lc, 1.0, 1.0, 0.5)[0] is want
    # rate 1/4: L_a = -2, L_b = -1 -> Length_min = (-1 + 1/2)/(3/4) = -2/3
    assert orc.check_triple(-2.0, -1.0, -0.75, 1.0, 0.5, 0.25)[0] is True
    assert orc.check_triple(-2.0, -1.0, -0.625, 1.0, 0.5, 0.25)[0] is False
    # the part across the sample must not grow from the older iterate to the newer one
    assert orc.check_triple(0.0, 1.0, 1.5, 3.0, 3.0, 0.5)[0] is True
    assert orc.check_triple(0.0, 1.0, 1.5, 3.0, 3.5, 0.5)[0] is False
    # a contraction rate of 1 or more leaves no interval
    assert orc.check_triple(0.0, 1.0, 1.5, 4.0, 3.0, 1.0)[0] is False
    assert orc.check_triple(0.0, 1.0, 1.5, 4.0, 3.0, 1.5)[0] is False
    # how close the decision was: (2 - 1.5)/2 against the interval, 1/4 against the perpendicular parts
    assert orc.check_triple(0.0, 1.0, 1.5, 4.0, 3.0, 0.5)[1] == 0.25
    assert orc.check_triple(0.0, 1.0, 1.9375, 4.0, 1.0, 0.5)[1] == 0.03125


def test_delay_server_hand_case():
    """x = (1, 0), y = +1, hinge, w_0 = (0, 1), tau = 1, every sample the same row; exact binary
    fractions throughout.  beta^2 = 1, so rate = eta*lambda + eta.

    eta = 1/2, lambda = 1/4 (rate 5/8):
      w_1 = w_0 - w_0/8 + x/2 = (1/2, 7/8), accepted (no triple yet).
      w_2: gradient at w_0 (margin 0): w_1 - w_0/8 + x/2 = (1, 3/4).  Triple projections 0, 1/2, 1;
           Length_min = (1/2)/(3/8) = 4/3, 1 lies in [1/2, 4/3]; perpendicular parts 1 -> 7/8.  Accepted.
      w_3: gradient at w_1 (margin 1/2): w_2 - w_1/8 + x/2 = (23/16, 41/64).  Projections 1/2, 1, 23/16;
           Length_min = (1 - 5/16)/(3/8) = 11/6; inside.  Accepted.
      w_4: gradient at w_2 (margin 1, slope 0): w_3 - w_2/8 = (21/16, 35/64).  Projections 1, 23/16, 21/16;
           the interval is [23/16, 13/6] and 21/16 is below it: rejected, and so is every later sample,
           because a rejected candidate leaves the server as it was.
    eta = 1/4, lambda = 1/2 (rate 3/8):
      w_1 = (1/4, 7/8); w_2 candidate (1/2, 3/4): Length_min = (1/4)/(5/8) = 2/5 < 1/2: rejected for good."""
    X = np.array([[1.0, 0.0]], dtype=np.float32)
    y = np.array([1.0], dtype=np.float32)
    want = {1: [0.5, 0.875], 2: [1.0, 0.75], 3: [1.4375, 0.640625]}
    for n in (1, 2, 3, 4, 9):
        w, accepted, _ = orc.delay_sgd(orc.Dense(X), y, [0] * n, 0.5, 0.25, orc.HINGE, 1, w0=[0.0, 1.0])
        assert accepted == min(n, 3) and w.tolist() == want[min(n, 3)]
    for n in (1, 2, 7):
        w, accepted, _ = orc.delay_sgd(orc.Dense(X), y, [0] * n, 0.25, 0.5, orc.HINGE, 1, w0=[0.0, 1.0])
        assert accepted == 1 and w.tolist() == [0.25, 0.875]
    # without the Check function nothing is thrown away
    w, accepted, _ = orc.delay_sgd(orc.Dense(X), y, [0] * 4, 0.5, 0.25, orc.HINGE, 1, w0=[0.0, 1.0], check=False)
    assert accepted == 4 and w.tolist() == [1.3125, 0.546875]


def test_first_call_of_check_looks_at_the_older_iterates_along_the_new_sample():
    """Rows a = (1, 0) and b = (0, 1), hinge, start 0, eta = 1/2, lambda = 1/4, tau = 2 (rate sqrt(5/8)).
    Two visits of a give w_1 = (1/2, 0), w_2 = (1, 0): the second passes because 1 lies between 1/2 and
    (1/2)/(1 - rate) > 2 and nothing is perpendicular to a.  Then b arrives.  Along b the three iterates
    w_0, w_1, w_2 all project to 0 while the part across b grew from 0 to 1/2: the first call rejects,
    before any candidate is formed.  With tau = 1 that call has only two iterates to look at and the
    sample is lost at the second call instead: projections 0, 0 leave the single point 0 and the
    candidate (15/16, 1/2) projects to 1/2."""
    X = np.array([[1.0, 0.0], [0.0, 1.0]], dtype=np.float32)
    y = np.array([1.0, 1.0], dtype=np.float32)
    for tau in (2, 1):
        w, accepted, _ = orc.delay_sgd(orc.Dense(X), y, [0, 0, 1, 1, 1], 0.5, 0.25, orc.HINGE, tau)
        assert accepted == 2 and w.tolist() == [1.0, 0.0]


def _brute_force_delay_server(X, y, idx, eta, lam, loss, tau, w0):
    """Algorithms 3 and 4 with every iterate kept and the perpendicular parts formed as vectors."""
    hist, taken = [np.array(w0, dtype=np.float64)], []
    for j in idx:
        x, yy = X[j].astype(np.float64), float(y[j])
        J = len(hist) - 1
        old = hist[max(J - tau, 0)]
        yhat = float(old @ x)
        slope = (-yy if yy * yhat < 1.0 else 0.0) if loss == orc.HINGE else -yy / (1.0 + math.exp(yy * yhat))
        cand = hist[J] - eta * lam * old - eta * slope * x
        beta2 = float(x @ x)
        rate = (eta * lam + eta * beta2) ** (1.0 / max(tau, 1))

        def passes(a, b, c):
            if rate >= 1.0:
                return False
            La, Lb, Lc = float(a @ x), float(b @ x), float(c @ x)
            Lmin = (Lb - rate * La) / (1.0 - rate)
            across_a, across_b = a - La / beta2 * x, b - Lb / beta2 * x
            return min(Lmin, Lb) <= Lc <= max(Lmin, Lb) and not np.linalg.norm(across_b) > np.linalg.norm(across_a)

        window = hist[max(J - tau, 0):]
        ok = all(passes(*window[i:i + 3]) for i in range(len(window) - 2))
        if ok and J >= 1:
            ok = passes(hist[J - 1], hist[J], cand)
        taken.append(ok)
        if ok:
            hist.append(cand)
    return hist[-1], taken


@pytest.mark.parametrize("loss", [orc.HINGE, orc.LOGISTIC])
@pytest.mark.parametrize("tau", [0, 1, 2, 4])
def test_delay_server_against_brute_force(loss, tau):
    rng = np.random.default_rng(100 + tau)
    X, y = _aligned_rows(rng, 96, 12, 1e-2)
    seen = 0
    for eta, lam in ((0.5, 0.25), (0.9, 0.05), (0.25, 0.5)):
        for trial in range(4):
            w0 = 0.5 * rng.standard_normal(12)
            idx = orc.sample_indices(7 + trial, tau, 0, 300, 96)
            w, accepted, closest = orc.delay_sgd(orc.Dense(X), y, idx, eta, lam, loss, tau, w0=w0)
            if closest < 1e-9:
                continue                                     # a tie that rounding may break either way
            want, taken = _brute_force_delay_server(X, y, idx, eta, lam, loss, tau, w0)
            assert accepted == sum(taken)
            np.testing.assert_allclose(w, want, rtol=1e-11, atol=1e-13)
            # rejected samples leave no trace: the same server without Check, fed only the samples
            # that were taken, walks through the same iterates
            kept = [j for j, ok in zip(idx, taken) if ok]
            again, n_again, _ = orc.delay_sgd(orc.Dense(X), y, kept, eta, lam, loss, tau, w0=w0, check=False)
            assert n_again == accepted and again.tolist() == w.tolist()
            seen = max(seen, accepted)
    assert seen >= 5                                          # the cases do get past the first updates


def test_delay_servers_take_their_own_streams_and_phase_2_weights_by_accepted_updates():
    """Algorithm 3, phase 2: v = sum_i weight_i w_i with the weights of Eq. 8 on the number of updates
    each server has made."""
    rng = np.random.default_rng(31)
    X, y = _aligned_rows(rng, 64, 9, 1e-2)
    n = [40, 25, 0, 33]
    W, accepted, _ = orc.run_delay_chains(orc.Dense(X), y, n, 0.5, 0.25, orc.LOGISTIC, 12, 2, check=False)
    assert accepted.tolist() == n and not W[2].any()
    for i in (0, 1, 3):
        w, _, _ = orc.delay_sgd(orc.Dense(X), y, orc.sample_indices(12, i, 0, n[i], 64), 0.5, 0.25, orc.LOGISTIC, 2,
                                check=False)
        assert W[i].tolist() == w.tolist()
    a = orc.weights_rate(accepted, 1 - 0.5 * 0.25)
    np.testing.assert_allclose(orc.combine(W, a), sum(a[i] * W[i] for i in range(4)), rtol=1e-15)
