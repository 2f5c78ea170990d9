"""The entry point that allocates nothing: wpsgd_objective_static keeps its partial sums in the
library's own static device area instead of a caller's workspace.  Called through the C ABI,
twice in a row (the second call on a smaller input, so the area still holds the first call's
partial sums behind the ones in use), it must give the bits of wpsgd_objective and the oracle's
value to the bar of the objective tests.
"""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_1708_04801_amd import api
from paper_1708_04801_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _dense_case(m, d, seed, bf16=False):
    rng = np.random.default_rng(seed)
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    wvec = (rng.standard_normal(d) * 2).astype(np.float32)
    y = np.where(X @ wvec + 0.5 * rng.standard_normal(m) >= 0, 1.0, -1.0).astype(np.float32)
    data = wl.f32_to_bf16_bits(X) if bf16 else X
    return wl.Workload("static", wl.LOGISTIC, 0.1, 1e-3, 0, np.array([1], dtype=np.int64), y, m, d, dense=data), wvec


def _both_ways(w, wvec, lam, loss, out):
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    wg = torch.from_numpy(wvec).cuda()
    want = api.wpsgd_objective(X, y, wg, lam, loss)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    got = api.wpsgd_objective_static(X, y, wg, lam, loss, out)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before          # nothing was allocated on the device
    assert torch.equal(got, want), (got.tolist(), want.tolist())
    Xo = orc.CSR(w.row_ptr, w.col_idx, w.vals, w.d) if w.is_csr else orc.Dense(w.dense)
    obj, err = orc.objective(Xo, w.y, wvec.astype(np.float64), lam, loss)
    g = got.cpu().numpy()
    assert g[0] == pytest.approx(obj, rel=1e-11, abs=1e-13)
    assert abs(g[1] - err) <= 1.0 / w.m


@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_objective_from_the_static_area_twice_in_a_row(loss):
    out = torch.empty(2, dtype=torch.float64, device="cuda")
    big, wbig = _dense_case(20000, 512, 1)              # 2048 workgroups: every partial-sum slot in use
    small, wsmall = _dense_case(333, 512, 2)            # 84 workgroups: the rest keeps the first call's sums
    _both_ways(big, wbig, 0.02, loss, out)
    _both_ways(small, wsmall, 0.02, loss, out)
    _both_ways(big, wbig, 0.5, loss, out)
    bf, wbf = _dense_case(1500, 4100, 3, bf16=True)
    _both_ways(bf, wbf, 1e-3, loss, out)
    sp = wl.sparse_hinge(m=6000, d=1 << 15, k=2, n_median=10)
    rng = np.random.default_rng(5)
    wsp = (rng.standard_normal(sp.d) * (rng.random(sp.d) < 0.3)).astype(np.float32)
    _both_ways(sp, wsp, 1e-3, loss, out)
    _both_ways(small, wsmall, 0.02, loss, out)


def test_objective_static_rejects_bad_arguments():
    X = api.Matrix(4, 8, dense=torch.zeros((4, 8), dtype=torch.float32, device="cuda"))
    y = torch.ones(4, dtype=torch.float32, device="cuda")
    w = torch.zeros(8, dtype=torch.float32, device="cuda")
    out = torch.empty(3, dtype=torch.float64, device="cuda")
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_objective_static(X, y, w, -1.0, wl.HINGE, out[:2])
    assert e.value.status == api.INVALID_ARG
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_objective_static(X, y, w, 0.1, 7, out[:2])
    assert e.value.status == api.INVALID_ARG
    torch.cuda.synchronize()
