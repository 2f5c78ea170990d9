"""Host-side checks of libwpsgd.so that need no GPU: the library loads, exports every symbol the
header declares, and its pure-host entry points (weights, benefit condition, host sample stream,
planner, argument checks) agree with the oracle and with the paper's fixed values."""
import ctypes
import os
import re

import numpy as np
import pytest

from conftest import ROOT, golden_rows
from oracle import oracle as orc
from paper_1708_04801_amd import api


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "wpsgd.h")).read()
    declared = set(re.findall(r"\b(wpsgd_[a-z_]+)\s*\(", header))
    assert declared == set(api.EXPORTS)
    lib = ctypes.CDLL(api.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("row", golden_rows("weights_cases.txt"))
def test_weights_rate_golden(row):
    rate_s, n_s, a_s = row.split(";")
    n = [int(t) for t in n_s.split()]
    want = np.array([float(t) for t in a_s.split()])
    rtol = 1e-13 + (max(n) - min(n)) * 2.3e-16
    np.testing.assert_allclose(api.wpsgd_weights_rate(n, float(rate_s)), want, rtol=rtol)


def test_weights_match_oracle_and_reduce_to_uniform():
    rng = np.random.default_rng(0)
    for k in (1, 4, 64, 2048):
        n = rng.integers(0, 80000, size=k)
        for eta, lam in [(0.05, 1e-4), (0.1, 1e-5), (0.5, 0.5), (0.3, 0.0)]:
            np.testing.assert_allclose(api.wpsgd_weights(n, eta, lam), orc.weights(n, eta, lam),
                                       rtol=1e-11, atol=1e-300)
        assert np.array_equal(api.wpsgd_weights(np.full(k, 777), 0.05, 1e-4), np.full(k, 1.0 / k))
    np.testing.assert_allclose(api.wpsgd_weights([3, 1], 0.5, 0.5), [0.64, 0.36], rtol=1e-15)
    # a delay so long that rate^T underflows: the weight goes to zero, nothing is NaN
    a = api.wpsgd_weights([100000, 0], 0.5, 0.9)
    assert a.tolist() == [1.0, 0.0]


def test_benefit_margin_matches_oracle():
    assert api.wpsgd_benefit_margin([1000, 800, 600, 400], 1 - 1e-5) == pytest.approx(
        1.97605578468828733, rel=1e-12)
    assert api.wpsgd_benefit_margin([3, 1], 0.75) == pytest.approx(orc.benefit_margin([3, 1], 0.75), rel=1e-14)


def test_span_condition_matches_oracle_and_closed_forms():
    assert api.wpsgd_span_condition([50, 50, 50], 0.99) == pytest.approx(0.99 ** 50, rel=1e-13)
    assert api.wpsgd_span_condition([10, 3, 0, 7], 0.97) == pytest.approx(4 / sum(0.97 ** -d for d in (10, 3, 0, 7)), rel=1e-13)
    for n, r in (([1000, 800, 600, 400], 1 - 1e-5), ([3, 1], 0.75), ([0, 0, 9], 1.0)):
        assert api.wpsgd_span_condition(n, r) == pytest.approx(orc.span_condition(n, r), rel=1e-13)
    for bad in (lambda: api.wpsgd_span_condition([3, -1], 0.9), lambda: api.wpsgd_span_condition([3, 1], 0.0),
                lambda: api.wpsgd_span_condition([3, 1], 1.5)):
        with pytest.raises(api.WpsgdError) as err:
            bad()
        assert err.value.status == api.INVALID_ARG


@pytest.mark.parametrize("row", golden_rows("sample_index_streams.txt"))
def test_host_sample_stream_golden(row):
    head, tail = row.split(":")
    seed, chain, m, n0 = (int(t) for t in head.split())
    want = [int(t) for t in tail.split()]
    assert api.wpsgd_sample_indices(seed, chain, n0, len(want), m).tolist() == want


def test_host_sample_stream_equals_oracle_bit_for_bit():
    for seed, chain, m in [(0, 0, 4096), (123456789012345, 77, 1000003), (2 ** 64 - 1, 2 ** 31 - 1, 2 ** 32 - 1),
                           (5, 1, 1)]:
        for n0 in (0, 2 ** 32 - 70):
            got = api.wpsgd_sample_indices(seed, chain, n0, 200, m)
            assert np.array_equal(got, orc.sample_indices(seed, chain, n0, 200, m))


def test_host_shard_stream_equals_oracle_bit_for_bit():
    for seed, m, k in [(0, 4096, 4), (77, 1000003, 10), (2 ** 64 - 1, 65537, 64), (5, 1, 1), (9, 17, 17)]:
        for chain in {0, k // 2, k - 1}:
            for n0 in (0, 12345):
                got = api.wpsgd_shard_indices(seed, chain, k, n0, 300, m)
                assert np.array_equal(got, orc.shard_indices(seed, chain, k, n0, 300, m))
    with pytest.raises(api.WpsgdError):
        api.wpsgd_shard_indices(0, 0, 5, 0, 1, 4)          # more nodes than rows


def test_argument_errors_are_reported_not_crashed():
    for bad in [lambda: api.wpsgd_weights([1, -2], 0.1, 0.1), lambda: api.wpsgd_weights([1], 0.0, 0.1),
                lambda: api.wpsgd_weights([1], 1.0, 1.0), lambda: api.wpsgd_weights([1], 0.1, -0.1),
                lambda: api.wpsgd_weights_rate([1], 1.5), lambda: api.wpsgd_weights_rate([1], 0.0),
                lambda: api.wpsgd_sample_indices(0, 0, 0, 4, 0), lambda: api.wpsgd_sample_indices(0, 0, 0, 4, 2 ** 32),
                lambda: api.wpsgd_sample_indices(0, -1, 0, 4, 10)]:
        with pytest.raises(api.WpsgdError) as err:
            bad()
        assert err.value.status == api.INVALID_ARG
    assert api.load().wpsgd_strerror(api.UNSUPPORTED).decode().startswith("no kernel")
    assert "gave up" in api.load().wpsgd_strerror(api.INCOMPLETE).decode()


class _FakeMatrix(api.Matrix):
    """A matrix descriptor with made-up device addresses: good enough for the planner, which
    never dereferences them."""

    def __init__(self, m, d, dtype=api.F32, ld=None, csr=False, base=0x10000):
        super().__init__(m, d)
        self._c = api._CMatrix()
        self._c.m, self._c.d = m, d
        if csr:
            self._c.row_ptr, self._c.col_idx, self._c.vals = base, base, base
        else:
            self._c.dense, self._c.ld, self._c.dtype = base, (ld or d), dtype

    def c_struct(self):
        return self._c


def test_planner_picks_registers_when_the_vector_fits_and_hbm_otherwise():
    d = api.wpsgd_describe_plan
    assert d(_FakeMatrix(4096, 64), 4, api.HINGE).startswith("dense_reg f32 hinge nt=64 ept=1 vec=1")
    assert "nt=64 ept=4 vec=4" in d(_FakeMatrix(1 << 20, 256), 2048, api.HINGE)
    assert "nt=256 ept=16 vec=4" in d(_FakeMatrix(262144, 4096), 64, api.LOGISTIC)
    assert "dense_reg bf16 logistic" in d(_FakeMatrix(65536, 65536, api.BF16), 32, api.LOGISTIC)
    assert "state=registers" in d(_FakeMatrix(65536, 65536, api.BF16), 32, api.LOGISTIC)
    assert d(_FakeMatrix(100, 1 << 20), 2, api.LOGISTIC).startswith("dense_mem")
    assert "hbm-f64" in d(_FakeMatrix(100, 1 << 20), 2, api.HINGE)
    assert "vec=1" in d(_FakeMatrix(100, 255), 2, api.HINGE)            # ragged d: scalar loads
    assert "vec=1" in d(_FakeMatrix(100, 256, base=0x10004), 2, api.HINGE)   # misaligned base
    assert d(_FakeMatrix(1000, 1 << 20, csr=True), 2, api.HINGE).startswith("csr")
    assert "dense_mem" in d(_FakeMatrix(100, 256), 2, api.HINGE, plan={"state_in_hbm": 1})
    with pytest.raises(api.WpsgdError) as err:
        d(_FakeMatrix(100, 256), 2, api.HINGE, plan={"threads": 64, "block_steps": 8})
    assert err.value.status == api.UNSUPPORTED
    # few fp32 logistic chains of 16 KiB rows: two steps per reduction round, helpers on the idle compute units
    few = d(_FakeMatrix(262144, 4096), 64, api.LOGISTIC)
    assert "B=2 P=4" in few and "helpers=2" in few
    many = d(_FakeMatrix(262144, 4096), 2048, api.LOGISTIC)
    assert "B=1 P=8" in many and "helpers" not in many
    assert "helpers=2" in d(_FakeMatrix(262144, 4096), 63, api.LOGISTIC)
    assert "helpers=1" in d(_FakeMatrix(262144, 4096), 128, api.LOGISTIC)            # one spare compute unit per chain
    assert "helpers" not in d(_FakeMatrix(262144, 4096), 129, api.LOGISTIC)
    assert "helpers" not in d(_FakeMatrix(262144, 4096), 64, api.LOGISTIC, plan={"helpers": -1})
    # rows too long for one 256-thread workgroup and compute units to spare: column slices
    assert "ept=32 vec=8 B=2 P=4" in d(_FakeMatrix(65536, 65536, api.BF16), 32, api.LOGISTIC)
    assert "slices=8" in d(_FakeMatrix(65536, 65536, api.BF16), 32, api.LOGISTIC)
    assert "ept=64 vec=8 B=2 P=2" in d(_FakeMatrix(65536, 65536, api.BF16), 33, api.LOGISTIC)    # 33 * 8 > 256 compute units:
    assert "slices=4" in d(_FakeMatrix(65536, 65536, api.BF16), 33, api.LOGISTIC)                # four wider slices
    assert "rows=lds" in d(_FakeMatrix(65536, 65536, api.BF16), 200, api.LOGISTIC)               # none to spare
    assert "slices=8" in d(_FakeMatrix(65536, 65536, api.BF16), 32, api.HINGE)          # fp64 state: no one-workgroup shape
    assert d(_FakeMatrix(65536, 65536, api.BF16), 200, api.HINGE).startswith("dense_mem")
    assert "slices=5" in d(_FakeMatrix(1000, 40000), 9, api.HINGE)                      # 5 * 8192 columns cover 40000, 4 do not
    assert "slices" not in d(_FakeMatrix(262144, 4096), 64, api.LOGISTIC)
    for bad in ({"helpers": 4}, {"helpers": -2}, {"rows": 5}, {"slices": 9}, {"slices": -1}):
        with pytest.raises(api.WpsgdError) as err:
            d(_FakeMatrix(262144, 4096), 64, api.LOGISTIC, plan=bad)
        assert err.value.status == api.INVALID_ARG


def test_planner_shapes_cover_the_row_for_any_size():
    """Whatever d, k, storage and loss: a register plan's lanes cover every column, a sliced plan
    leaves no slice empty and never asks for more workgroups than the device has compute units,
    and everything else falls to the kernel that keeps the model in HBM."""
    import re
    d_values = [1, 63, 64, 65, 255, 1000, 4096, 4100, 8192, 12000, 16384, 20000, 32768, 40000, 65536, 70000, 131072, 200000]
    for dtype in (api.F32, api.BF16):
        for loss in (api.HINGE, api.LOGISTIC):
            for k in (1, 9, 32, 33, 64, 129, 3000):
                for d in d_values:
                    if dtype == api.BF16 and d % 8:
                        continue
                    text = api.wpsgd_describe_plan(_FakeMatrix(1 << 16, d, dtype), k, loss)
                    if text.startswith("dense_mem"):
                        continue
                    f = {m.group(1): int(m.group(2)) for m in re.finditer(r"(nt|ept|vec|B|P|slices|helpers)=(\d+)", text)}
                    slices = f.get("slices", 1)
                    assert f["nt"] * f["ept"] * slices >= d, (text, d, k)
                    assert slices == 1 or f["nt"] * f["ept"] * (slices - 1) < d, (text, d, k)
                    assert k * slices + k * f.get("helpers", 0) <= 256 or (slices == 1 and "helpers" not in f), (text, d, k)
                    assert 64 % (f["B"] * max(f["P"], 1)) == 0, (text, d, k)
                    assert not ("slices" in f and "helpers" in f), (text, d, k)


def test_workspace_sizes():
    # status block + chain order + step counts + stream offsets + share descriptions + progress counters
    # (256-byte slots) + power table (1 KiB) + shuffled row order (4 bytes a row) + room for the model vectors in HBM
    assert api.wpsgd_run_chains_workspace(_FakeMatrix(4096, 64), 4, api.HINGE) == 2560 + 4096 * 4 + 4 * 64 * 8
    ws = api.wpsgd_run_chains_workspace(_FakeMatrix(1000, 1 << 20, csr=True), 128, api.HINGE)
    assert ws >= 128 * (1 << 20) * 8
    ws = api.wpsgd_run_chains_workspace(_FakeMatrix(1000, 1 << 20, csr=True), 128, api.LOGISTIC)
    assert 128 * (1 << 20) * 4 <= ws < 128 * (1 << 20) * 4 + 4096 + 4 * 1000 + 2048 + 1024 + 256
    assert api.wpsgd_combine_workspace(64, 4096) == 512
    # delay servers: the sample counts, then max(tau, 1) + 2 vectors of d doubles per server, then 32 bytes per row
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(4096, 64), 4, 0) == 256 + 4 * 3 * 64 * 8 + 4096 * 32
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(4096, 64), 4, 1) == 256 + 4 * 3 * 64 * 8 + 4096 * 32
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(4096, 100), 40, 16) == 512 + 40 * 18 * 100 * 8 + 4096 * 32
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(3, 64), 1, 2) == 256 + 4 * 64 * 8 + 256
    # what the call would refuse has no size: a negative or too long delay, no servers, sparse rows
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(4096, 64), 4, -1) == 0
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(4096, 64), 4, 17) == 0
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(4096, 64), 0, 2) == 0
    assert api.wpsgd_run_delay_chains_workspace(_FakeMatrix(4096, 64, csr=True), 4, 2) == 0
    # spans: what the chains need, then the chains' models, then what the average needs
    fm = _FakeMatrix(4096, 64)
    assert api.wpsgd_run_spans_workspace(fm, 4, api.HINGE) == \
        api.wpsgd_run_chains_workspace(fm, 4, api.HINGE) + 1024 + 256
