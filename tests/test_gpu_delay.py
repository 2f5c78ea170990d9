"""GPU parity of the delay-SGD servers (Section IV, Algorithms 3 and 4) against the fp64 CPU oracle.

Both sides compute in fp64 and differ only in the order of their sums, so:
  * the number of accepted updates per server is compared exactly;
  * every server's last iterate (fp32 on the GPU, rounded once) to a relative L2 error of 1e-6;
  * a server whose oracle run came within 1e-12 (relative) of a tie in some comparison of the Check
    function is exempt from both, because there rounding decides; the tests bound how many those are.
    (A dot product of d <= 4096 fp64 terms is good to about d * 2^-53 = 5e-13 in the worst case and to
    a few 1e-16 typically; a server makes thousands of comparisons, so its closest one is often near
    1e-9 by chance, which is why the bar is not wider.)
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_1708_04801_amd import api
from paper_1708_04801_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-6
TIE = 1e-12


def rel_l2(got, want):
    denom = np.linalg.norm(want)
    return np.linalg.norm(got.astype(np.float64) - want) / (denom if denom > 0 else 1.0)


def run_both(w, tau, check, start=True, loss=None):
    loss = w.loss if loss is None else loss
    w_start = w.meta["w_start"] if start else None
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    Wg, acc_g = api.wpsgd_run_delay_chains(X, y, w.n_steps, w.eta, w.lam, loss, w.seed, tau, check=check,
                                           w_start=None if w_start is None else torch.from_numpy(w_start).cuda())
    torch.cuda.synchronize()
    Wo = np.zeros((w.k, w.d))
    acc_o = np.zeros(w.k, dtype=np.int64)
    gap = np.zeros(w.k)
    for i in range(w.k):
        idx = orc.sample_indices(w.seed, i, 0, int(w.n_steps[i]), w.m)
        Wo[i], acc_o[i], gap[i] = orc.delay_sgd(orc.Dense(w.dense), w.y, idx, w.eta, w.lam, loss, tau,
                                                w0=None if w_start is None else w_start.astype(np.float64), check=check)
    return Wg.cpu().numpy(), acc_g.cpu().numpy(), Wo, acc_o, gap


def compare(Wg, acc_g, Wo, acc_o, gap, label, max_ties=0):
    assert np.isfinite(Wg).all(), label
    tied = gap < TIE
    assert tied.sum() <= max_ties, f"{label}: {tied.sum()} servers within {TIE} of a tie"
    clear = ~tied
    assert np.array_equal(acc_g[clear], acc_o[clear]), f"{label}: accepted {acc_g.tolist()} against {acc_o.tolist()}"
    errs = np.array([rel_l2(Wg[i], Wo[i]) for i in range(Wo.shape[0])])
    assert (errs[clear] <= TOL).all(), f"{label}: servers off by {errs.tolist()}"


@pytest.mark.parametrize("tau", [0, 1, 2, 3, 4, 7, 16])
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
@pytest.mark.parametrize("d", [1003, 1024, 2560])
def test_plain_delay_sgd(tau, loss, d):
    """check = 0: every candidate is kept.  Ragged width (scalar loads) and aligned widths (tau + 1 samples
    per exchange for delays 1 to 4), sample counts that are no multiple of tau + 1, idle server, zero start."""
    w = wl.delay_servers(m=512, d=d, k=5, n_lo=40, n_hi=90, tau=tau, loss=loss, spread=0.3, data_seed=50 + tau)
    w.n_steps[3] = 0
    Wg, acc_g, Wo, acc_o, gap = run_both(w, tau, check=False, start=(tau % 2 == 0))
    assert acc_g.tolist() == w.n_steps.tolist()
    compare(Wg, acc_g, Wo, acc_o, gap, f"plain tau={tau}")


@pytest.mark.parametrize("tau", [0, 1, 2, 3, 4, 5, 16])
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
@pytest.mark.parametrize("d,bf16", [(1024, False), (777, False), (2048, True), (330, True)])
def test_servers_under_check(tau, loss, d, bf16):
    w = wl.delay_servers(m=1024, d=d, k=12, n_lo=300, n_hi=900, tau=tau, loss=loss, bf16=bf16,
                         data_seed=7 * tau + d)
    Wg, acc_g, Wo, acc_o, gap = run_both(w, tau, check=True)
    compare(Wg, acc_g, Wo, acc_o, gap, f"check tau={tau} d={d}", max_ties=1)
    assert acc_o.max() >= 4 and (acc_o < w.n_steps).all()      # samples are taken and samples are thrown away


@pytest.mark.parametrize("tau", [0, 1, 3, 4])
@pytest.mark.parametrize("d,bf16", [(4096, False), (3584, True)])
def test_servers_under_check_on_rows_of_the_measured_width(tau, d, bf16):
    w = wl.delay_servers(m=2048, d=d, k=6, n_lo=500, n_hi=1500, tau=tau, bf16=bf16, data_seed=90 + tau)
    Wg, acc_g, Wo, acc_o, gap = run_both(w, tau, check=True)
    compare(Wg, acc_g, Wo, acc_o, gap, f"check tau={tau} d={d}", max_ties=1)
    Wg, acc_g, Wo, acc_o, gap = run_both(w, tau, check=False)
    compare(Wg, acc_g, Wo, acc_o, gap, f"plain tau={tau} d={d}")


@pytest.mark.parametrize("tau", [0, 1, 2, 4])
@pytest.mark.parametrize("d", [8, 64, 2048])
def test_few_samples_and_narrow_rows(tau, d):
    """Servers with 0 to 11 samples (less than a batch, one more than a batch, ...) on rows that fill only
    a few lanes or every lane of the widest eight-element shape; one data row only for the last server's
    stream to repeat."""
    w = wl.delay_servers(m=96, d=d, k=12, n_lo=1, n_hi=2, tau=tau, spread=0.05, data_seed=200 + tau + d)
    w.n_steps[:] = np.arange(12)
    for check in (True, False):
        Wg, acc_g, Wo, acc_o, gap = run_both(w, tau, check=check)
        compare(Wg, acc_g, Wo, acc_o, gap, f"few samples tau={tau} d={d} check={check}", max_ties=2)
    one = wl.delay_servers(m=1, d=d, k=3, n_lo=5, n_hi=9, tau=tau, data_seed=9)
    compare(*run_both(one, tau, check=False), f"one row tau={tau} d={d}")


@pytest.mark.parametrize("tau", [0, 2, 4])
def test_servers_that_visit_few_of_many_rows(tau):
    """When the servers together visit less than a quarter of the rows, no table of per-row quantities is
    built and every sample is decided on its own (another kernel than in the cases above)."""
    w = wl.delay_servers(m=16384, d=1024, k=3, n_lo=300, n_hi=900, tau=tau, data_seed=70 + tau)
    assert 4 * w.n_steps.sum() < w.m
    Wg, acc_g, Wo, acc_o, gap = run_both(w, tau, check=True)
    compare(Wg, acc_g, Wo, acc_o, gap, f"few visits tau={tau}", max_ties=1)
    assert acc_o.max() >= 4


def test_check_from_the_zero_start_of_algorithm_3():
    """From w_0 = 0 nothing lies across the second sample yet while w_1 does, so the second update passes
    only for a sample parallel to the first, and then the comparison of the two parts is a tie."""
    w = wl.delay_servers(m=1024, d=512, k=8, n_lo=200, n_hi=400, tau=2, data_seed=3)
    Wg, acc_g, Wo, acc_o, gap = run_both(w, 2, check=True, start=False)
    compare(Wg, acc_g, Wo, acc_o, gap, "zero start", max_ties=w.k)
    assert (acc_o[gap >= TIE] == 1).all() and (acc_g >= 1).all()


@pytest.mark.parametrize("d", [1024, 1001])
def test_rows_too_long_for_a_contraction_are_all_rejected_after_the_first(d):
    """eta*lambda + eta*|x|^2 >= 1 leaves no interval: once there is a triple to test nothing passes, but
    the first update has none and is made."""
    w = wl.delay_servers(m=256, d=d, k=4, n_lo=20, n_hi=60, tau=2, data_seed=17)
    w.dense *= np.float32(3.0)
    Wg, acc_g, Wo, acc_o, gap = run_both(w, 2, check=True)
    assert acc_o.tolist() == [1, 1, 1, 1]
    compare(Wg, acc_g, Wo, acc_o, gap, f"long rows d={d}")


def test_hand_worked_servers():
    """The two servers worked by hand for the oracle's pins (exact binary fractions), through the GPU."""
    X = api.Matrix(1, 2, dense=torch.tensor([[1.0, 0.0]], device="cuda"))
    y = torch.tensor([1.0], device="cuda")
    start = torch.tensor([0.0, 1.0], device="cuda")
    want = {1: [0.5, 0.875], 2: [1.0, 0.75], 3: [1.4375, 0.640625]}
    n = [1, 2, 3, 4, 9]
    W, acc = api.wpsgd_run_delay_chains(X, y, n, 0.5, 0.25, wl.HINGE, 0, 1, w_start=start)
    assert acc.tolist() == [1, 2, 3, 3, 3]
    assert W.tolist() == [want[min(v, 3)] for v in n]
    W, acc = api.wpsgd_run_delay_chains(X, y, [1, 2, 7], 0.25, 0.5, wl.HINGE, 0, 1, w_start=start)
    assert acc.tolist() == [1, 1, 1] and W.tolist() == [[0.25, 0.875]] * 3
    W, acc = api.wpsgd_run_delay_chains(X, y, [4], 0.5, 0.25, wl.HINGE, 0, 1, check=False, w_start=start)
    assert acc.tolist() == [4] and W.tolist() == [[1.3125, 0.546875]]


def test_phase_2_weights_the_servers_by_their_accepted_updates():
    w = wl.delay_servers(m=2048, d=1024, k=16, n_lo=100, n_hi=800, tau=2, data_seed=11)
    Wg, acc_g, Wo, acc_o, gap = run_both(w, 2, check=True)
    compare(Wg, acc_g, Wo, acc_o, gap, "phase 2", max_ties=1)
    if (gap < TIE).any():
        pytest.skip("a server sits on a tie")
    rate = 1.0 - w.eta * w.lam
    a = api.wpsgd_weights_rate(acc_g, rate)
    np.testing.assert_allclose(a, orc.weights_rate(acc_o, rate), rtol=1e-12)
    v = api.wpsgd_combine(torch.from_numpy(Wg).cuda(), a).cpu().numpy()
    assert rel_l2(v, orc.combine(Wo, orc.weights_rate(acc_o, rate))) <= TOL


def test_full_size_servers():
    """The measured configuration: 128 servers, rows of 4096 fp32, delay 2, every server compared."""
    w = wl.delay_servers()
    Wg, acc_g, Wo, acc_o, gap = run_both(w, w.meta["tau"], check=True)
    compare(Wg, acc_g, Wo, acc_o, gap, "full size", max_ties=2)
    Wg, acc_g, Wo, acc_o, gap = run_both(w, w.meta["tau"], check=False)
    compare(Wg, acc_g, Wo, acc_o, gap, "full size, no check")


def test_refusals():
    w = wl.delay_servers(m=64, d=32, k=2, n_lo=5, n_hi=9, data_seed=1)
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    for tau, status in ((-1, api.INVALID_ARG), (17, api.UNSUPPORTED)):
        with pytest.raises(api.WpsgdError) as e:
            api.wpsgd_run_delay_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, 0, tau,
                                       workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
        assert e.value.status == status
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_run_delay_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, 0, 2,
                                   workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.WORKSPACE_TOO_SMALL
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_run_delay_chains(X, y, [-1, 3], w.eta, w.lam, w.loss, 0, 2)
    assert e.value.status == api.INVALID_ARG
    sparse = wl.sparse_hinge(m=64, d=256, k=2, nnz_mean=8, n_median=10)
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_run_delay_chains(api.matrix_from_workload(sparse), torch.from_numpy(sparse.y).cuda(), [3, 3],
                                   0.1, 0.1, wl.HINGE, 0, 2,
                                   workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.UNSUPPORTED
    assert api.wpsgd_run_delay_chains_workspace(X, 2, 2) == 256 + 2 * 4 * 32 * 8 + 64 * 32
    assert api.wpsgd_run_delay_chains_workspace(X, 2, 17) == 0
