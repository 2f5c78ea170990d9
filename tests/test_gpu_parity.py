"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle, element by
element on the same seeded inputs.

Bars (fp32 GPU output against the fp64 oracle):
  * sample-index streams: bit-exact;
  * final weighted model and every chain's model: relative L2 error <= 1e-4;
  * hinge chains whose oracle run came within 1e-9 of the kink y*yhat = 1 are reported and
    exempted from the per-chain check (the branch there is decided by rounding), never from the
    check of the final model.
Small cases cover every kernel family and forced plan, ragged and unaligned shapes, idle
chains, heavy shrink; the five full-size workloads compare every chain and the final model.
"""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_1708_04801_amd import api
from paper_1708_04801_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-4
KINK = 1e-9


def rel_l2(got, want):
    denom = np.linalg.norm(want)
    return np.linalg.norm(got.astype(np.float64) - want) / (denom if denom > 0 else 1.0)


def oracle_matrix(w):
    return orc.CSR(w.row_ptr, w.col_idx, w.vals, w.d) if w.is_csr else orc.Dense(w.dense)


def gpu_chains(w, plan=None, X=None, y=None):
    X = api.matrix_from_workload(w) if X is None else X
    y = torch.from_numpy(w.y).cuda() if y is None else y
    W = api.wpsgd_run_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed, plan=plan)
    torch.cuda.synchronize()
    return W


def check_against_oracle(w, W_gpu, chain_ids=None, label="", csr_mode=orc.PLAIN):
    """Per-chain and final-model parity; chain_ids selects the chains the oracle computes.
    csr_mode = orc.LAZY runs sparse chains in the oracle's scalar-scale mode (pinned to the literal
    shrink at 1e-12 by the CPU tests), for matrices so wide that the literal shrink takes minutes."""
    ids = np.arange(w.k) if chain_ids is None else np.asarray(chain_ids)
    Wo, margin = orc.run_chains(oracle_matrix(w), w.y, w.n_steps, w.eta, w.lam, w.loss, w.seed,
                                chain_ids=ids, csr_mode=csr_mode)
    Wg = W_gpu[torch.from_numpy(ids).cuda()].cpu().numpy()
    assert np.isfinite(Wg).all(), f"{label}: non-finite model"
    errs = np.array([rel_l2(Wg[q], Wo[q]) for q in range(ids.size)])
    ambiguous = (margin < KINK) if w.loss == wl.HINGE else np.zeros(ids.size, dtype=bool)
    bad = (errs > TOL) & ~ambiguous
    assert not bad.any(), (f"{label}: chains {ids[bad].tolist()} off by {errs[bad].tolist()} "
                           f"(closest approach to the hinge kink: {margin[bad].tolist()})")
    if chain_ids is None:
        a = orc.weights(w.n_steps, w.eta, w.lam)
        v_ref = orc.combine(Wo, a)
        a_gpu = api.wpsgd_weights(w.n_steps, w.eta, w.lam)
        np.testing.assert_allclose(a_gpu, a, rtol=1e-11)
        v_gpu = api.wpsgd_combine(W_gpu, a_gpu).cpu().numpy()
        err = rel_l2(v_gpu, v_ref)
        assert err <= TOL, f"{label}: final model off by {err} (min margin {margin.min()})"
    return errs, margin


# ------------------------------------------------------------------ sample stream, bit-exact

@pytest.mark.parametrize("seed,chain,n0,count,m", [
    (0, 0, 0, 1000, 4096), (0, 3, 0, 777, 1000000), (7, 5, 123, 4097, 1000003),
    (2 ** 64 - 1, 2 ** 31 - 1, 2 ** 32 - 100, 300, 2 ** 32 - 1), (1, 0, 5, 0, 10), (1, 2047, 63, 2, 1)])
def test_device_sample_stream_is_bit_exact(seed, chain, n0, count, m):
    got = api.wpsgd_sample_indices_device(seed, chain, n0, count, m).cpu().numpy()
    assert np.array_equal(got, orc.sample_indices(seed, chain, n0, count, m))
    assert np.array_equal(got, api.wpsgd_sample_indices(seed, chain, n0, count, m))


# ------------------------------------------------------------------ combine

@pytest.mark.parametrize("k,d", [(1, 1), (4, 64), (3, 1023), (64, 4096), (128, 40000), (300, 77),
                                 (2048, 256), (17, 262144 + 4), (1000, 5)])
def test_combine_matches_oracle(k, d):
    rng = np.random.default_rng(k * 1000003 + d)
    W = rng.standard_normal((k, d)).astype(np.float32)
    a = rng.random(k)
    a /= a.sum()
    got = api.wpsgd_combine(torch.from_numpy(W).cuda(), a).cpu().numpy()
    want = orc.combine(W.astype(np.float64), a)
    # fp64 accumulation, one rounding to fp32 at the end
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-30)
    e = np.zeros(k)
    e[k // 2] = 1.0
    assert np.array_equal(api.wpsgd_combine(torch.from_numpy(W).cuda(), e).cpu().numpy(), W[k // 2])


def test_combine_unaligned_views():
    rng = np.random.default_rng(5)
    base = torch.from_numpy(rng.standard_normal(6 * 100 + 1).astype(np.float32)).cuda()
    W = base[1:].view(6, 100)                # 4-byte aligned only
    a = rng.random(6)
    got = api.wpsgd_combine(W, a).cpu().numpy()
    np.testing.assert_allclose(got, orc.combine(W.cpu().numpy().astype(np.float64), a), rtol=2e-7)


# ------------------------------------------------------------------ chains, small cases

def test_tiny_hinge_workload_full_path():
    """The smallest workload at its stated size: 4 chains of 1000/800/600/400 steps, d = 64."""
    w = wl.tiny_hinge()
    errs, margin = check_against_oracle(w, gpu_chains(w), label="tiny_hinge")
    assert errs.max() < 1e-6          # fp64 state: only the final rounding to fp32 remains


DENSE_PLANS = [
    # (d, loss, plan)
    (64, wl.HINGE, None), (64, wl.LOGISTIC, {"block_steps": 4}), (100, wl.HINGE, None),
    (128, wl.LOGISTIC, None), (255, wl.LOGISTIC, None), (256, wl.HINGE, None),
    (256, wl.HINGE, {"prefetch": 16}), (256, wl.LOGISTIC, {"block_steps": 2}),
    (256, wl.HINGE, {"block_steps": 4}), (252, wl.LOGISTIC, None),
    (1000, wl.LOGISTIC, None), (1024, wl.HINGE, {"block_steps": 4}), (2048, wl.LOGISTIC, {"block_steps": 4}),
    (3000, wl.LOGISTIC, None), (3001, wl.HINGE, None), (4096, wl.LOGISTIC, None),
    (4096, wl.LOGISTIC, {"block_steps": 1, "prefetch": 8}), (4096, wl.LOGISTIC, {"block_steps": 2, "prefetch": 4}),
    (4096, wl.HINGE, {"block_steps": 1, "prefetch": 4}), (4096, wl.HINGE, {"block_steps": 4}),
    (4096, wl.LOGISTIC, {"threads": 512}), (4096, wl.LOGISTIC, {"threads": 1024, "block_steps": 1}),
    (4099, wl.LOGISTIC, None), (8192, wl.HINGE, None), (8000, wl.LOGISTIC, {"block_steps": 4}),
    (12000, wl.LOGISTIC, None), (16384, wl.HINGE, None), (20000, wl.LOGISTIC, None),
    (4096, wl.LOGISTIC, {"state_in_hbm": 1}), (300, wl.HINGE, {"state_in_hbm": 1}),
    (5001, wl.HINGE, {"state_in_hbm": 1}), (20000, wl.LOGISTIC, {"state_in_hbm": 1, "threads": 1024}),
    (70000, wl.LOGISTIC, None), (40000, wl.HINGE, None),
    # long rows: next row staged in LDS (the default up to 128 KiB) or streamed twice
    (12000, wl.LOGISTIC, {"rows": 3}), (16384, wl.HINGE, {"rows": 3}), (20000, wl.LOGISTIC, {"rows": 3}),
    (20000, wl.HINGE, {"rows": 2}), (32768, wl.LOGISTIC, {"rows": 2}), (32768, wl.HINGE, None),
    (40000, wl.LOGISTIC, None),
]


@pytest.mark.parametrize("d,loss,plan", DENSE_PLANS)
def test_dense_fp32_chains(d, loss, plan):
    rng = np.random.default_rng(d * 7 + loss)
    m, k = 512, 9
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    wstar = rng.standard_normal(d)
    y = np.where(X @ wstar + 0.3 * rng.standard_normal(m) >= 0, 1.0, -1.0).astype(np.float32)
    n = np.array([257, 64, 0, 1, 130, 63, 300, 5, 128], dtype=np.int64)
    w = wl.Workload("dense_small", loss, 0.5 if loss == wl.HINGE else 2.0, 1e-3, 11, n, y, m, d, dense=X)
    Xg = api.matrix_from_workload(w)
    desc = api.wpsgd_describe_plan(Xg, k, loss, plan)
    if plan and "rows" in plan:
        assert {2: "rows=lds", 3: "rows=twice"}[plan["rows"]] in desc
    W = gpu_chains(w, plan=plan, X=Xg)
    check_against_oracle(w, W, label=f"d={d} [{desc}]")
    assert (W[2] == 0).all()                                     # idle chain keeps w_0 = 0
    W2 = gpu_chains(w, plan=plan, X=Xg)
    assert torch.equal(W, W2)                                    # same inputs, same bits


@pytest.mark.parametrize("k,d,helpers,extra", [
    (8, 4096, 3, {}), (16, 4096, 1, {}), (8, 2048, 2, {}), (24, 8192, 0, {}), (8, 1000, 3, {}),
    (9, 4096, 2, {}), (13, 4096, 3, {"block_steps": 1}), (70, 2048, 1, {}), (3, 4096, 3, {"block_steps": 2})])
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_dense_chains_with_helper_workgroups(k, d, helpers, extra, loss):
    """Workgroups that run ahead of the chains and pull their rows into L2 change when a row arrives,
    never what is computed: same bits as without them, and the oracle's result."""
    rng = np.random.default_rng(k * 31 + d + loss)
    m = 700
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = rng.integers(0, 400, size=k).astype(np.int64)
    n[0], n[1] = 0, 1
    w = wl.Workload("helped", loss, 0.3, 1e-3, 5, n, y, m, d, dense=X)
    Xg = api.matrix_from_workload(w)
    plan = {"threads": 256, "helpers": helpers, **extra}
    desc = api.wpsgd_describe_plan(Xg, k, loss, plan)
    assert (f"helpers={helpers}" if helpers else "helpers=2") in desc
    W = gpu_chains(w, plan=plan, X=Xg)
    assert torch.equal(W, gpu_chains(w, plan={"threads": 256, "helpers": -1, **extra}, X=Xg))
    check_against_oracle(w, W, label=f"helped k={k} d={d} [{desc}]")


@pytest.mark.parametrize("d,bf16,loss,plan", [
    (4096, False, wl.LOGISTIC, {"slices": 2}), (4096, False, wl.LOGISTIC, {"slices": 4}),
    (4096, False, wl.LOGISTIC, {"slices": 2, "block_steps": 1}), (4096, False, wl.HINGE, {"slices": 2}),
    (4096, False, wl.HINGE, {"slices": 4}), (3000, False, wl.LOGISTIC, {"slices": 3}),
    (8192, False, wl.LOGISTIC, {"slices": 8}), (5000, False, wl.HINGE, {"slices": 5}),
    (4096, True, wl.LOGISTIC, {"slices": 2}), (16384, True, wl.HINGE, {"slices": 4}),
    (65536, True, wl.LOGISTIC, {"slices": 4}), (65536, True, wl.LOGISTIC, {"slices": 8}),
    (4096, False, wl.LOGISTIC, {"slices": 2, "block_steps": 4}), (4096, False, wl.HINGE, {"slices": 4, "block_steps": 2}),
    (65536, True, wl.LOGISTIC, {"slices": 8, "block_steps": 4}), (65536, True, wl.LOGISTIC, {"slices": 4, "block_steps": 4}),
    (16384, True, wl.HINGE, {"slices": 2, "block_steps": 2}), (4096, False, wl.HINGE, {"slices": 2, "block_steps": 1}),
    (16384, False, wl.HINGE, None), (32768, True, wl.HINGE, None)])
def test_dense_chains_cut_into_column_slices(d, bf16, loss, plan):
    """A chain spread over several compute units, each with a slice of the columns; the slices add
    their partial sums through global memory once per round."""
    rng = np.random.default_rng(d + 11 * loss + (plan["slices"] if plan else 0))
    m, k = 160, 6
    Xf = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    n = np.array([257, 64, 0, 1, 130, 63], dtype=np.int64)
    if bf16:
        bits = wl.f32_to_bf16_bits(Xf)
        y = np.where(wl.bf16_bits_to_f32(bits) @ rng.standard_normal(d) >= 0, 1.0, -1.0).astype(np.float32)
        w = wl.Workload("sliced_bf16", loss, 0.5, 1e-3, 13, n, y, m, d, dense=bits)
    else:
        y = np.where(Xf @ rng.standard_normal(d) + 0.3 * rng.standard_normal(m) >= 0, 1.0, -1.0).astype(np.float32)
        w = wl.Workload("sliced", loss, 0.5 if loss == wl.HINGE else 2.0, 1e-3, 13, n, y, m, d, dense=Xf)
    Xg = api.matrix_from_workload(w)
    desc = api.wpsgd_describe_plan(Xg, k, loss, plan)
    assert (f"slices={plan['slices']}" if plan else "slices=8") in desc           # few chains of long rows are cut by default
    W = gpu_chains(w, plan=plan, X=Xg)
    check_against_oracle(w, W, label=f"sliced d={d} [{desc}]")
    assert (W[2] == 0).all()
    assert torch.equal(W, gpu_chains(w, plan=plan, X=Xg))            # same inputs, same bits


def _wide_case(seed, k=32, d=65536, m=200, n_hi=260):
    rng = np.random.default_rng(seed)
    Xf = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    bits = wl.f32_to_bf16_bits(Xf)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = rng.integers(40, n_hi, size=k).astype(np.int64)
    return wl.Workload("wide_pair", wl.LOGISTIC, 0.5, 1e-3, seed, n, y, m, d, dense=bits)


def test_two_sliced_launches_on_two_streams_at_once():
    """Two default launches of few wide chains (each cut into as many column slices as the device has
    compute units for) queued on two streams at the same time: the slices of a chain wait for each
    other, so the two launches must not end up half seated each.  Both match the oracle."""
    wa, wb = _wide_case(101), _wide_case(202)
    Xa, Xb = api.matrix_from_workload(wa), api.matrix_from_workload(wb)
    assert "slices=8" in api.wpsgd_describe_plan(Xa, wa.k, wa.loss)
    ya, yb = torch.from_numpy(wa.y).cuda(), torch.from_numpy(wb.y).cuda()
    ws_a = torch.empty(api.wpsgd_run_chains_workspace(Xa, wa.k, wa.loss), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(api.wpsgd_run_chains_workspace(Xb, wb.k, wb.loss), dtype=torch.uint8, device="cuda")
    Wa = torch.empty((wa.k, wa.d), dtype=torch.float32, device="cuda")
    Wb = torch.empty((wb.k, wb.d), dtype=torch.float32, device="cuda")
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(3):                 # several pairs back to back, so that launches do meet on the device
        api.wpsgd_run_chains(Xa, ya, wa.n_steps, wa.eta, wa.lam, wa.loss, wa.seed, W=Wa, workspace=ws_a, stream=sa)
        api.wpsgd_run_chains(Xb, yb, wb.n_steps, wb.eta, wb.lam, wb.loss, wb.seed, W=Wb, workspace=ws_b, stream=sb)
    assert api.wpsgd_chains_status(ws_a, stream=sa) == api.OK
    assert api.wpsgd_chains_status(ws_b, stream=sb) == api.OK
    torch.cuda.synchronize()
    check_against_oracle(wa, Wa, label="sliced pair, first stream")
    check_against_oracle(wb, Wb, label="sliced pair, second stream")


@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_slices_that_give_up_say_so(loss):
    """The give-up path of sliced chains, forced from the host: with no time to wait, every slice
    loses the others at its first exchange.  Every kernel still ends by itself; the rows of the chains
    that took steps are NaN through and through, idle chains are untouched, the status word reports
    it, and the next ordinary call on the same workspace is clean again."""
    rng = np.random.default_rng(31 + loss)
    m, d, k = 120, 8192, 5
    Xf = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = np.array([90, 0, 33, 64, 1], dtype=np.int64)
    w = wl.Workload("gave_up", loss, 0.5, 1e-3, 3, n, y, m, d, dense=Xf)
    X = api.matrix_from_workload(w)
    yg = torch.from_numpy(w.y).cuda()
    ws = torch.empty(api.wpsgd_run_chains_workspace(X, k, loss, {"slices": 4}), dtype=torch.uint8, device="cuda")
    W = api.wpsgd_run_chains(X, yg, n, w.eta, w.lam, loss, w.seed, workspace=ws, plan={"slices": 4, "slice_wait_us": -1})
    assert api.wpsgd_chains_status(ws) == api.INCOMPLETE
    Wh = W.cpu().numpy()
    for i in range(k):
        assert np.isnan(Wh[i]).all() if n[i] > 0 else (Wh[i] == 0).all(), f"chain {i}"
    W = api.wpsgd_run_chains(X, yg, n, w.eta, w.lam, loss, w.seed, workspace=ws, plan={"slices": 4})
    assert api.wpsgd_chains_status(ws) == api.OK
    check_against_oracle(w, W, label="after a give-up")
    # periodic averaging keeps the verdict of every span
    spans_ws = torch.empty(api.wpsgd_run_spans_workspace(X, k, loss, {"slices": 4}), dtype=torch.uint8, device="cuda")
    api.wpsgd_run_spans(X, yg, np.array([20, 10, 5, 20, 0]), 3, w.eta, w.lam, loss, w.seed, workspace=spans_ws,
                        plan={"slices": 4})
    assert api.wpsgd_chains_status(spans_ws) == api.OK
    v = api.wpsgd_run_spans(X, yg, np.array([20, 10, 5, 20, 0]), 3, w.eta, w.lam, loss, w.seed, workspace=spans_ws,
                            plan={"slices": 4, "slice_wait_us": -1})
    assert api.wpsgd_chains_status(spans_ws) == api.INCOMPLETE
    assert torch.isnan(v).all()


BF16_PLANS = [(64, None), (256, None), (512, None), (520, None), (2048, {"block_steps": 4}), (4096, None),
              (8192, {"block_steps": 1}), (16384, None), (30000, None), (65536, None),
              (65536, {"state_in_hbm": 1}), (4100, {"state_in_hbm": 1}), (40000, None), (33000, None),
              (16384, {"rows": 3}), (30000, {"rows": 3}), (12000, {"rows": 2})]


@pytest.mark.parametrize("d,plan", BF16_PLANS)
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_dense_bf16_chains(d, plan, loss):
    rng = np.random.default_rng(d * 13 + loss)
    m = 96
    Xf = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    bits = wl.f32_to_bf16_bits(Xf)
    wstar = rng.standard_normal(d)
    y = np.where(wl.bf16_bits_to_f32(bits) @ wstar >= 0, 1.0, -1.0).astype(np.float32)
    n = np.array([70, 0, 33, 129], dtype=np.int64)
    w = wl.Workload("bf16_small", loss, 0.5, 1e-3, 3, n, y, m, d, dense=bits)
    Xg = api.matrix_from_workload(w)
    desc = api.wpsgd_describe_plan(Xg, 4, loss, plan)
    check_against_oracle(w, gpu_chains(w, plan=plan, X=Xg), label=f"bf16 d={d} [{desc}]")


def test_widest_bf16_rows_both_ways():
    """d = 65536 in bfloat16 (128 KiB rows): few chains are cut into column slices, one workgroup per
    chain means the LDS-staged kernel, the kernel that streams every row twice stays reachable; all
    must match the oracle."""
    rng = np.random.default_rng(77)
    m, d = 80, 65536
    bits = wl.f32_to_bf16_bits((rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32))
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = np.array([200, 65, 1, 0, 64], dtype=np.int64)
    w = wl.Workload("bf16_widest", wl.LOGISTIC, 0.5, 1e-3, 5, n, y, m, d, dense=bits)
    Xg = api.matrix_from_workload(w)
    assert "slices=8" in api.wpsgd_describe_plan(Xg, 5, wl.LOGISTIC)                 # few chains: eight compute units each
    assert "rows=lds" in api.wpsgd_describe_plan(Xg, 5, wl.LOGISTIC, {"slices": 1})
    assert "rows=lds" in api.wpsgd_describe_plan(Xg, 200, wl.LOGISTIC)               # no compute units to spare
    assert "rows=twice" in api.wpsgd_describe_plan(Xg, 5, wl.LOGISTIC, {"rows": 3})
    for plan in (None, {"slices": 1}, {"rows": 3}):
        W = gpu_chains(w, plan=plan, X=Xg)
        check_against_oracle(w, W, label=f"bf16 widest {plan}")
        assert torch.equal(W, gpu_chains(w, plan=plan, X=Xg))
    # fp64 state (hinge) has no one-workgroup register shape at this width: slices, or the HBM-state kernel
    wh = wl.Workload("bf16_widest_hinge", wl.HINGE, 0.5, 1e-3, 5, n, y, m, d, dense=bits)
    assert "slices=8" in api.wpsgd_describe_plan(Xg, 5, wl.HINGE)
    assert "dense_mem" in api.wpsgd_describe_plan(Xg, 200, wl.HINGE)
    for plan in (None, {"slices": 4}):
        W = gpu_chains(wh, plan=plan, X=Xg)
        check_against_oracle(wh, W, label=f"bf16 widest hinge {plan}")
        assert torch.equal(W, gpu_chains(wh, plan=plan, X=Xg))


def test_dense_rows_with_padding_and_misaligned_base():
    rng = np.random.default_rng(21)
    m, d, ld = 200, 300, 304
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = np.array([100, 40], dtype=np.int64)
    w = wl.Workload("padded", wl.LOGISTIC, 1.0, 1e-2, 5, n, y, m, d, dense=X)
    padded = torch.zeros((m, ld), dtype=torch.float32, device="cuda")
    padded[:, :d] = torch.from_numpy(X).cuda()
    Xg = api.Matrix(m, d, dense=padded[:, :d])                     # ld = 304, 16-byte aligned rows
    assert "vec=4" in api.wpsgd_describe_plan(Xg, 2, wl.LOGISTIC)
    check_against_oracle(w, gpu_chains(w, X=Xg), label="padded rows")
    flat = torch.zeros(m * d + 1, dtype=torch.float32, device="cuda")
    flat[1:] = torch.from_numpy(X).cuda().reshape(-1)
    Xu = api.Matrix(m, d, dense=flat[1:].view(m, d))               # base only 4-byte aligned
    assert "vec=1" in api.wpsgd_describe_plan(Xu, 2, wl.LOGISTIC)
    check_against_oracle(w, gpu_chains(w, X=Xu), label="misaligned base")


@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_heavy_shrink_folds_the_scale(loss):
    """(1 - eta*lambda)^n far below fp32 range: the lazy scale must be folded back in time."""
    rng = np.random.default_rng(33)
    m, d = 64, 256
    X = rng.standard_normal((m, d)).astype(np.float32) / 16
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = np.array([900, 333], dtype=np.int64)
    w = wl.Workload("shrink", loss, 0.5, 0.6, 2, n, y, m, d, dense=X)      # rate 0.7, 0.7^900 ~ 1e-140
    for plan in (None, {"threads": 256}, {"state_in_hbm": 1}):
        check_against_oracle(w, gpu_chains(w, plan=plan), label=f"heavy shrink {plan}")


def test_single_chain_and_equal_lengths():
    w = wl.tiny_hinge(n_steps=(500,))
    W = gpu_chains(w)
    v = api.wpsgd_combine(W, api.wpsgd_weights(w.n_steps, w.eta, w.lam))
    assert torch.equal(v, W[0])                                   # k = 1: weight 1
    w = wl.tiny_hinge(n_steps=(200, 200, 200))
    W = gpu_chains(w)
    a = api.wpsgd_weights(w.n_steps, w.eta, w.lam)
    assert np.array_equal(a, np.full(3, 1 / 3))                   # Algorithm 2's plain average
    v = api.wpsgd_combine(W, a).cpu().numpy()
    np.testing.assert_allclose(v, W.cpu().numpy().astype(np.float64).mean(axis=0), rtol=3e-7, atol=1e-12)


def test_all_chains_idle():
    w = wl.tiny_hinge(n_steps=(0, 0, 0))
    W = gpu_chains(w)
    assert (W == 0).all()
    v = api.wpsgd_combine(W, api.wpsgd_weights(w.n_steps, w.eta, w.lam))
    assert (v == 0).all()


def test_many_more_chains_than_compute_units():
    w = wl.many_chains(m=8192, d=256, k=3000, n_full=60)
    check_against_oracle(w, gpu_chains(w), label="3000 chains")


# ------------------------------------------------------------------ CSR chains

# The three sparse kernels: two waves per chain (the default), one wave with head columns in LDS, plain.
SPARSE_PLANS = [None, {"prefetch": 4}, {"prefetch": 1}]
SPARSE_TAGS = {None: "P=8", 4: "P=4", 1: "P=1"}
CACHED_PLANS = [None, {"prefetch": 4}]


def _sparse_tag(plan):
    return SPARSE_TAGS[plan["prefetch"] if plan else None]


@pytest.mark.parametrize("plan", SPARSE_PLANS)
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_sparse_chains_small(loss, plan):
    w = wl.sparse_hinge(m=5000, d=1 << 14, k=12, n_median=300)
    w.loss = loss
    w.n_steps[3] = 0
    w.n_steps[5] = 1
    X = api.matrix_from_workload(w)
    desc = api.wpsgd_describe_plan(X, w.k, loss, plan)
    assert _sparse_tag(plan) in desc
    W = gpu_chains(w, plan=plan, X=X)
    check_against_oracle(w, W, label=f"sparse small [{desc}]")
    assert torch.equal(W, gpu_chains(w, plan=plan, X=X))


@pytest.mark.parametrize("plan", CACHED_PLANS)
def test_sparse_tail_conflicts_are_caught(plan):
    """Few tail columns and many steps: consecutive steps keep writing the columns the next
    ones have already fetched, so the stale-value check has to fire all the time."""
    rng = np.random.default_rng(45)
    m, d = 300, 8192 + 40                       # 40 columns beyond the LDS-resident head
    rp, ci, va = [0], [], []
    for r in range(m):
        head = np.sort(rng.choice(8192, size=20, replace=False))
        tail = 8192 + np.sort(rng.choice(40, size=6, replace=False))
        c = np.concatenate([head, tail])
        v = rng.standard_normal(c.size)
        v /= np.linalg.norm(v)
        ci += c.tolist()
        va += v.tolist()
        rp.append(len(ci))
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    for loss in (wl.HINGE, wl.LOGISTIC):
        w = wl.Workload("tail_conflicts", loss, 0.3, 1e-4, 9, np.array([900, 257, 64, 3], dtype=np.int64), y, m, d,
                        row_ptr=np.array(rp, dtype=np.int64), col_idx=np.array(ci, dtype=np.int32),
                        vals=np.array(va, dtype=np.float32))
        check_against_oracle(w, gpu_chains(w, plan=plan), label=f"tail conflicts {plan}")


@pytest.mark.parametrize("plan", CACHED_PLANS)
@pytest.mark.parametrize("period", [1, 3, 7, 8, 9, 12, 16])
def test_sparse_tail_conflicts_at_a_fixed_distance(period, plan):
    """Tail columns that come back exactly every `period` steps: model values fetched ahead of
    time are stale for short periods (the stale-value check must fire) and must be fresh for
    long ones (the check does not fire, the early fetch must already see the last write)."""
    m, n_steps, seed = 4096, 700, 17
    visits = api.wpsgd_sample_indices(seed, 0, 0, n_steps, m)
    first = {}
    for t, r in enumerate(visits.tolist()):
        first.setdefault(r, t)
    rng = np.random.default_rng(period)
    d = 8192 + 3 * period + 8
    rp, ci, va = [0], [], []
    for r in range(m):
        cols = np.sort(rng.choice(8192, size=10, replace=False)).tolist()
        if r in first:
            cols += [8192 + 3 * (first[r] % period) + q for q in range(3)]
        v = rng.standard_normal(len(cols))
        v /= np.linalg.norm(v)
        ci += cols
        va += v.tolist()
        rp.append(len(ci))
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    for loss in (wl.HINGE, wl.LOGISTIC):
        w = wl.Workload("tail_period", loss, 0.4, 1e-4, seed, np.array([n_steps], dtype=np.int64), y, m, d,
                        row_ptr=np.array(rp, dtype=np.int64), col_idx=np.array(ci, dtype=np.int32),
                        vals=np.array(va, dtype=np.float32))
        X = api.matrix_from_workload(w)
        assert _sparse_tag(plan) in api.wpsgd_describe_plan(X, 1, loss, plan)
        check_against_oracle(w, gpu_chains(w, X=X, plan=plan), label=f"tail period {period} {plan}")


def test_sparse_heavy_shrink_takes_the_plain_kernel():
    w = wl.sparse_hinge(m=2000, d=1 << 13, k=4, n_median=400)
    w.eta, w.lam = 0.5, 0.6                      # rate 0.7: the lazy scale must be folded
    X = api.matrix_from_workload(w)
    check_against_oracle(w, gpu_chains(w, X=X), label="sparse heavy shrink")


@pytest.mark.parametrize("plan", SPARSE_PLANS)
def test_sparse_rows_longer_than_the_register_window(plan):
    rng = np.random.default_rng(44)
    m, d = 40, 20000
    rp, ci, va = [0], [], []
    for r in range(m):
        nnz = [1, 64, 65, 256, 257, 700][r % 6]
        c = np.sort(rng.choice(d, size=nnz, replace=False))
        v = rng.standard_normal(nnz)
        v /= np.linalg.norm(v)
        ci += c.tolist()
        va += v.tolist()
        rp.append(len(ci))
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    w = wl.Workload("long_rows", wl.HINGE, 0.3, 1e-2, 9, np.array([150, 80, 0], dtype=np.int64), y, m, d,
                    row_ptr=np.array(rp, dtype=np.int64), col_idx=np.array(ci, dtype=np.int32),
                    vals=np.array(va, dtype=np.float32))
    for loss in (wl.HINGE, wl.LOGISTIC):
        w.loss = loss
        check_against_oracle(w, gpu_chains(w, plan=plan), label=f"long sparse rows {plan}")


# ------------------------------------------------------------------ start vector and stream offsets

def _oracle_from(w, w_start, offsets):
    """Every chain by the oracle's single-chain routine on an explicit index stream."""
    Xo = orc.CSR(w.row_ptr, w.col_idx, w.vals, w.d) if w.is_csr else orc.Dense(w.dense)
    W = np.zeros((w.k, w.d))
    closest = np.inf
    for i in range(w.k):
        idx = orc.sample_indices(w.seed, i, int(offsets[i]), int(w.n_steps[i]), w.m)
        W[i], mm = orc.sgd(Xo, w.y, idx, w.eta, w.lam, w.loss, w0=w_start.astype(np.float64))
        closest = min(closest, mm)
    return W, closest


def _check_from(w, plan, label):
    rng = np.random.default_rng(w.d + w.k)
    w_start = (rng.standard_normal(w.d) * 0.5).astype(np.float32)
    offsets = rng.integers(0, 500, size=w.k).astype(np.int64)
    offsets[0] = 0
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    W = api.wpsgd_run_chains_from(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed,
                                  w_start=torch.from_numpy(w_start).cuda(), step_offsets=offsets, plan=plan)
    Wo, closest = _oracle_from(w, w_start, offsets)
    if w.loss == wl.HINGE:
        assert closest > KINK, f"{label}: a hinge step sits on the kink ({closest:.3e})"
    Wg = W.cpu().numpy().astype(np.float64)
    for i in range(w.k):
        err = np.linalg.norm(Wg[i] - Wo[i]) / max(np.linalg.norm(Wo[i]), 1e-300)
        assert err <= TOL, f"{label}: chain {i} rel L2 {err:.3e}"
    # the defaults reproduce wpsgd_run_chains bit for bit
    assert torch.equal(api.wpsgd_run_chains_from(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed, plan=plan),
                       api.wpsgd_run_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed, plan=plan))


@pytest.mark.parametrize("d,plan", [(64, None), (300, None), (4096, None), (4096, {"block_steps": 4}),
                                    (5000, {"state_in_hbm": 1}), (20000, None), (20000, {"rows": 3})])
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_dense_chains_from_a_start_vector_and_stream_offsets(d, plan, loss):
    rng = np.random.default_rng(d + 3 * loss)
    m = 300
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = np.array([130, 0, 64, 7], dtype=np.int64)
    w = wl.Workload("from_dense", loss, 0.3, 1e-2, 21, n, y, m, d, dense=X)
    _check_from(w, plan, f"dense d={d} {plan}")


@pytest.mark.parametrize("plan", SPARSE_PLANS)
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_sparse_chains_from_a_start_vector_and_stream_offsets(loss, plan):
    w = wl.sparse_hinge(m=3000, d=1 << 14, k=5, n_median=150)
    w.loss = loss
    w.n_steps[1] = 0
    _check_from(w, plan, f"sparse {plan}")


def test_bf16_chains_from_a_start_vector():
    rng = np.random.default_rng(8)
    m, d = 64, 65536
    bits = wl.f32_to_bf16_bits((rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32))
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    w = wl.Workload("from_bf16", wl.LOGISTIC, 0.5, 1e-3, 5, np.array([70, 3], dtype=np.int64), y, m, d, dense=bits)
    _check_from(w, None, "bf16 widest")


def test_periodic_averaging_restarts_chains_from_the_weighted_average():
    """Two spans of unequal chains with a weighted average in between (Section III, Deduction 2),
    each chain continuing its own sample stream: device path against the oracle."""
    w = wl.tiny_hinge()
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    n1, n2 = w.n_steps // 2, w.n_steps - w.n_steps // 2
    W1 = api.wpsgd_run_chains(X, y, n1, w.eta, w.lam, w.loss, w.seed)
    v1 = api.wpsgd_combine(W1, api.wpsgd_weights(n1, w.eta, w.lam))
    W2 = api.wpsgd_run_chains_from(X, y, n2, w.eta, w.lam, w.loss, w.seed, w_start=v1, step_offsets=n1)
    v2 = api.wpsgd_combine(W2, api.wpsgd_weights(n2, w.eta, w.lam)).cpu().numpy()
    Xo = orc.Dense(w.dense)
    Wo1, _ = orc.run_chains(Xo, w.y, n1, w.eta, w.lam, w.loss, w.seed)
    vo1 = orc.combine(Wo1, orc.weights(n1, w.eta, w.lam))
    Wo2 = np.zeros_like(Wo1)
    for i in range(w.k):
        idx = orc.sample_indices(w.seed, i, int(n1[i]), int(n2[i]), w.m)
        Wo2[i], _ = orc.sgd(Xo, w.y, idx, w.eta, w.lam, w.loss, w0=vo1)
    vo2 = orc.combine(Wo2, orc.weights(n2, w.eta, w.lam))
    assert np.linalg.norm(v2 - vo2) / np.linalg.norm(vo2) <= TOL


def _check_spans(w, steps, n_spans, label, sampling=0, start=None, plan=None):
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    Xo = orc.CSR(w.row_ptr, w.col_idx, w.vals, w.d) if w.is_csr else orc.Dense(w.dense)
    w0 = None if start is None else torch.from_numpy(start).cuda()
    v = api.wpsgd_run_spans(X, y, steps, n_spans, w.eta, w.lam, w.loss, w.seed, w_start=w0, sampling=sampling, plan=plan)
    torch.cuda.synchronize()
    vo = orc.run_spans(Xo, w.y, steps, n_spans, w.eta, w.lam, w.loss, w.seed,
                       w0=None if start is None else start.astype(np.float64), shards=sampling == api.SAMPLE_SHARDS)
    err = rel_l2(v.cpu().numpy(), vo)
    assert err <= TOL, f"{label}: after {n_spans} spans rel L2 {err:.3e}"
    return v


def test_span_averaging_entry_point_matches_the_oracle():
    """wpsgd_run_spans (Section III, Deduction 2) against the oracle's loop over its own single-chain
    routine: dense and sparse rows, both losses and sampling schemes, a start vector, idle chains."""
    w = wl.tiny_hinge()
    _check_spans(w, [50, 40, 30, 20], 5, "tiny hinge")
    _check_spans(w, [50, 40, 30, 20], 3, "tiny hinge on shards", sampling=api.SAMPLE_SHARDS)
    rng = np.random.default_rng(12)
    m, d = 400, 4096
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(X @ rng.standard_normal(d) >= 0, 1.0, -1.0).astype(np.float32)
    wd = wl.Workload("spans_dense", wl.LOGISTIC, 0.5, 1e-2, 9, np.array([64, 0, 33, 64, 7], dtype=np.int64), y, m, d, dense=X)
    start = (0.1 * rng.standard_normal(d)).astype(np.float32)
    v = _check_spans(wd, wd.n_steps, 4, "dense logistic from a start vector", start=start)
    # one span is the whole of Algorithm 1; the output may overwrite the start vector
    Xg, yg = api.matrix_from_workload(wd), torch.from_numpy(wd.y).cuda()
    one = api.wpsgd_run_spans(Xg, yg, wd.n_steps, 1, wd.eta, wd.lam, wd.loss, wd.seed)
    W = api.wpsgd_run_chains(Xg, yg, wd.n_steps, wd.eta, wd.lam, wd.loss, wd.seed)
    assert torch.equal(one, api.wpsgd_combine(W, api.wpsgd_weights(wd.n_steps, wd.eta, wd.lam)))
    buf = torch.from_numpy(start).cuda()
    api.wpsgd_run_spans(Xg, yg, wd.n_steps, 4, wd.eta, wd.lam, wd.loss, wd.seed, w_start=buf, w_out=buf)
    assert torch.equal(buf, v)
    ws = wl.sparse_hinge(m=3000, d=1 << 14, k=5, n_median=150)
    for loss in (wl.HINGE, wl.LOGISTIC):
        ws.loss = loss
        _check_spans(ws, np.minimum(ws.n_steps, 120), 3, f"sparse loss {loss}")
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_run_spans(Xg, yg, wd.n_steps, 0, wd.eta, wd.lam, wd.loss, wd.seed)
    assert e.value.status == api.INVALID_ARG
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_run_spans(Xg, yg, [0, 0, 0], 2, wd.eta, wd.lam, wd.loss, wd.seed)
    assert e.value.status == api.INVALID_ARG


def test_run_chains_from_rejects_negative_offsets():
    w = wl.tiny_hinge()
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_run_chains_from(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed, step_offsets=[0, -1, 0, 0])
    assert e.value.status == api.INVALID_ARG


# ------------------------------------------------------------------ streams

def test_calls_on_side_streams_match_the_default_stream():
    """The library queues on the caller's stream and keeps no device state of its own: the whole path on
    two side streams at once (separate outputs and workspaces) gives the bits of the default stream."""
    rng = np.random.default_rng(44)
    m, d = 300, 1000
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    cases = [wl.Workload("side_a", wl.LOGISTIC, 0.5, 1e-2, 3, np.array([200, 90, 0, 150], dtype=np.int64), y, m, d, dense=X),
             wl.Workload("side_b", wl.HINGE, 0.1, 1e-3, 4, np.array([64, 300, 17], dtype=np.int64), y, m, d, dense=X)]
    Xg, yg = api.matrix_from_workload(cases[0]), torch.from_numpy(y).cuda()

    def whole_path(w, stream=None):
        W = api.wpsgd_run_chains(Xg, yg, w.n_steps, w.eta, w.lam, w.loss, w.seed, stream=stream)
        v = api.wpsgd_combine(W, api.wpsgd_weights(w.n_steps, w.eta, w.lam), stream=stream)
        spans = api.wpsgd_run_spans(Xg, yg, np.minimum(w.n_steps, 40), 3, w.eta, w.lam, w.loss, w.seed, stream=stream)
        return W, v, spans

    want = [whole_path(w) for w in cases]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    got = []
    for w, st in zip(cases, streams):
        with torch.cuda.stream(st):                       # torch allocates the outputs on that stream too
            got.append(whole_path(w, stream=st))
    for st in streams:
        st.synchronize()
    for g, wnt in zip(got, want):
        for a_, b_ in zip(g, wnt):
            assert torch.equal(a_, b_)
    check_against_oracle(cases[0], got[0][0], label="side stream")


def test_two_host_threads_call_the_library_at_once():
    """The staging buffers for host arrays belong to the calling thread: two threads, each on a stream
    of its own, run the whole path side by side many times and get the single-threaded bits."""
    import threading
    rng = np.random.default_rng(45)
    m, d = 256, 512
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    cases = [wl.Workload("thread_a", wl.LOGISTIC, 0.5, 1e-2, 3, np.array([120, 60, 90, 7, 33], dtype=np.int64), y, m, d, dense=X),
             wl.Workload("thread_b", wl.HINGE, 0.1, 1e-3, 4, np.array([64, 100, 17], dtype=np.int64), y, m, d, dense=X)]
    Xg, yg = api.matrix_from_workload(cases[0]), torch.from_numpy(y).cuda()

    def whole_path(w, stream=None):
        W = api.wpsgd_run_chains(Xg, yg, w.n_steps, w.eta, w.lam, w.loss, w.seed, stream=stream)
        return api.wpsgd_combine(W, api.wpsgd_weights(w.n_steps, w.eta, w.lam), stream=stream)

    want = [whole_path(w).clone() for w in cases]
    torch.cuda.synchronize()
    wrong, errors = [0, 0], []

    def worker(i):
        try:
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                for _ in range(40):
                    got = whole_path(cases[i], stream=st)
                    st.synchronize()
                    wrong[i] += int(not torch.equal(got, want[i]))
        except Exception as e:           # (an assertion in a thread would otherwise go unseen)
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert wrong == [0, 0]


# ------------------------------------------------------------------ random shapes and plans

def _random_case(rng):
    kind = rng.choice(["dense", "dense", "dense", "bf16", "csr"])
    loss = int(rng.integers(0, 2))
    k = int(rng.choice([1, 2, 3, 5, 8, 9, 16, 33]))
    d = int([rng.integers(1, 300), rng.integers(300, 5000), rng.integers(5000, 20000), rng.integers(20000, 70000),
             rng.choice([64, 256, 4096, 8192, 16384, 32768, 65536]), rng.integers(1, 70000)][rng.integers(0, 6)])
    if kind == "bf16" or rng.random() < 0.6:
        d = max(8, d // 8 * 8)
    m = int(rng.integers(max(k, 2), 400))
    n = rng.integers(0, 160, size=k).astype(np.int64)
    if rng.random() < 0.5:
        n[rng.integers(0, k)] = int(rng.integers(160, 400))
    eta, lam = float(rng.choice([0.5, 0.1, 0.02])), float(rng.choice([1e-2, 1e-3, 1e-5, 0.0]))
    seed = int(rng.integers(0, 2 ** 40))
    shards, use_start = bool(rng.random() < 0.25), bool(rng.random() < 0.3)
    plan, r = None, rng.random()
    if kind != "csr":
        if r < 0.15:
            plan = {"slices": int(rng.choice([2, 3, 4, 8]))}
        elif r < 0.25:
            plan = {"block_steps": int(rng.choice([1, 2, 4]))}
        elif r < 0.30:
            plan = {"helpers": int(rng.choice([1, 2, 3]))}
        elif r < 0.35:
            plan = {"helpers": -1}
        elif r < 0.40:
            plan = {"state_in_hbm": 1}
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    if kind == "csr":
        d = max(d, 64)
        rp, ci, va = [0], [], []
        for _ in range(m):
            ln = int(min(d, max(1, rng.poisson(20))))
            ci.append(np.sort(rng.choice(d, size=ln, replace=False)).astype(np.int32))
            vals = rng.standard_normal(ln).astype(np.float32)
            va.append(vals / max(np.linalg.norm(vals), 1e-6))
            rp.append(rp[-1] + ln)
        w = wl.Workload("random", loss, eta, lam, seed, n, y, m, d, row_ptr=np.array(rp, dtype=np.int64),
                        col_idx=np.concatenate(ci), vals=np.concatenate(va))
    else:
        X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
        w = wl.Workload("random", loss, eta, lam, seed, n, y, m, d, dense=wl.f32_to_bf16_bits(X) if kind == "bf16" else X)
    start = (0.3 * rng.standard_normal(d)).astype(np.float32) if use_start else None
    return w, plan, shards, start


@pytest.mark.parametrize("batch", range(4))
def test_random_shapes_plans_sampling_and_start_vectors(batch):
    """Seeded random cases (widths 1..70000, 1..33 chains, all storages, forced and default plans,
    both sampling schemes, with and without a start vector): every chain against the oracle."""
    ran = 0
    for it in range(40):
        rng = np.random.default_rng(7_000_003 * (batch + 1) + it)
        w, plan, shards, start = _random_case(rng)
        X = api.matrix_from_workload(w)
        try:
            desc = api.wpsgd_describe_plan(X, w.k, w.loss, plan)
        except api.WpsgdError as e:
            assert e.status == api.UNSUPPORTED            # a forced plan this shape has no kernel for
            continue
        W = api.wpsgd_run_chains_from(X, torch.from_numpy(w.y).cuda(), w.n_steps, w.eta, w.lam, w.loss, w.seed,
                                      w_start=None if start is None else torch.from_numpy(start).cuda(),
                                      sampling=api.SAMPLE_SHARDS if shards else 0, plan=plan)
        torch.cuda.synchronize()
        Wg = W.cpu().numpy().astype(np.float64)
        Xo = oracle_matrix(w)
        for i in range(w.k):
            idx = orc.shard_indices(w.seed, i, w.k, 0, int(w.n_steps[i]), w.m) if shards else \
                orc.sample_indices(w.seed, i, 0, int(w.n_steps[i]), w.m)
            wo, margin = orc.sgd(Xo, w.y, idx, w.eta, w.lam, w.loss, w0=None if start is None else start.astype(np.float64))
            label = f"case {batch}/{it} chain {i} d={w.d} k={w.k} plan={plan} shards={shards} [{desc}]"
            assert np.isfinite(Wg[i]).all(), label
            if w.loss == wl.HINGE and margin < KINK:
                continue
            assert rel_l2(Wg[i], wo) <= TOL, label
        ran += 1
    assert ran >= 25


# ------------------------------------------------------------------ partition-and-shuffle sampling

def test_device_shard_stream_is_bit_exact():
    for seed, m, k, chain in [(0, 4096, 4, 1), (3, 1000003, 128, 127), (11, 65537, 9, 0), (5, 70, 64, 33)]:
        for n0 in (0, 63, 1000):
            got = api.wpsgd_shard_indices_device(seed, chain, k, n0, 500, m).cpu().numpy()
            assert np.array_equal(got, orc.shard_indices(seed, chain, k, n0, 500, m))


def _check_shards(w, plan, label):
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    W = api.wpsgd_run_chains_from(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed, sampling=api.SAMPLE_SHARDS, plan=plan)
    Xo = orc.CSR(w.row_ptr, w.col_idx, w.vals, w.d) if w.is_csr else orc.Dense(w.dense)
    Wg = W.cpu().numpy().astype(np.float64)
    for i in range(w.k):
        idx = orc.shard_indices(w.seed, i, w.k, 0, int(w.n_steps[i]), w.m)
        wo, closest = orc.sgd(Xo, w.y, idx, w.eta, w.lam, w.loss)
        if w.loss == wl.HINGE and w.n_steps[i] > 0:
            assert closest > KINK, f"{label}: a hinge step sits on the kink"
        err = np.linalg.norm(Wg[i] - wo) / max(np.linalg.norm(wo), 1e-300)
        assert err <= TOL, f"{label}: chain {i} rel L2 {err:.3e}"


@pytest.mark.parametrize("d,plan", [(64, None), (300, None), (4096, None), (5000, {"state_in_hbm": 1}), (20000, None),
                                    (20000, {"rows": 3})])
@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_dense_chains_on_shuffled_shards(d, plan, loss):
    rng = np.random.default_rng(d + 5 * loss)
    m = 301
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = np.array([130, 0, 75, 200], dtype=np.int64)          # 200 > 75 rows per node: a second pass over the share
    w = wl.Workload("shards_dense", loss, 0.3, 1e-2, 21, n, y, m, d, dense=X)
    _check_shards(w, plan, f"dense d={d} {plan}")


@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
@pytest.mark.parametrize("plan", [{"threads": 256, "helpers": 2}, {"threads": 256, "helpers": 1, "block_steps": 1}])
def test_helped_chains_from_offsets_and_on_shards(plan, loss):
    """Helper workgroups walk the same sample stream as their chain under every sampling mode:
    a start vector with per-chain stream offsets, and partition-and-shuffle sampling."""
    rng = np.random.default_rng(17 + loss)
    m, d, k = 401, 4096, 8
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    y = np.where(rng.random(m) < 0.5, 1.0, -1.0).astype(np.float32)
    n = np.array([130, 0, 75, 200, 64, 1, 333, 90], dtype=np.int64)
    w = wl.Workload("helped_from", loss, 0.3, 1e-2, 21, n, y, m, d, dense=X)
    assert "helpers=" in api.wpsgd_describe_plan(api.matrix_from_workload(w), k, loss, plan)
    _check_from(w, plan, f"helped from {plan}")
    _check_shards(w, plan, f"helped shards {plan}")


@pytest.mark.parametrize("plan", SPARSE_PLANS)
def test_sparse_chains_on_shuffled_shards(plan):
    w = wl.sparse_hinge(m=3000, d=1 << 14, k=5, n_median=150)
    _check_shards(w, plan, f"sparse {plan}")


# ------------------------------------------------------------------ objective and error rate

def _check_objective(w, wvec, lam, label):
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    got = api.wpsgd_objective(X, y, torch.from_numpy(wvec).cuda(), lam, w.loss).cpu().numpy()
    Xo = orc.CSR(w.row_ptr, w.col_idx, w.vals, w.d) if w.is_csr else orc.Dense(w.dense)
    obj, err = orc.objective(Xo, w.y, wvec.astype(np.float64), lam, w.loss)
    assert got[0] == pytest.approx(obj, rel=1e-11, abs=1e-13), label
    assert abs(got[1] - err) <= 1.0 / w.m, label          # a row with y*yhat within rounding of 0 may flip


@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
@pytest.mark.parametrize("d", [1, 63, 64, 300, 512, 1000, 4096, 5000])
def test_objective_dense(d, loss):
    rng = np.random.default_rng(100 + d)
    m = 777
    X = (rng.standard_normal((m, d)) / math.sqrt(d)).astype(np.float32)
    wvec = rng.standard_normal(d).astype(np.float32) * 2
    y = np.where(X @ wvec + 0.5 * rng.standard_normal(m) >= 0, 1.0, -1.0).astype(np.float32)
    w = wl.Workload("obj", loss, 0.1, 1e-3, 0, np.array([1], dtype=np.int64), y, m, d, dense=X)
    _check_objective(w, wvec, 0.02, f"dense d={d}")
    _check_objective(w, np.zeros(d, dtype=np.float32), 0.5, f"dense d={d} w=0")     # log 2 or 1, every row wrong
    w16 = wl.Workload("obj16", loss, 0.1, 1e-3, 0, np.array([1], dtype=np.int64), y, m, d, dense=wl.f32_to_bf16_bits(X))
    _check_objective(w16, wvec, 0.02, f"bf16 d={d}")


@pytest.mark.parametrize("loss", [wl.HINGE, wl.LOGISTIC])
def test_objective_sparse_and_row_subsets(loss):
    w = wl.sparse_hinge(m=6000, d=1 << 15, k=2, n_median=10)
    w.loss = loss
    rng = np.random.default_rng(5)
    wvec = (rng.standard_normal(w.d) * (rng.random(w.d) < 0.3)).astype(np.float32)
    _check_objective(w, wvec, 1e-3, "sparse")
    # the last 1000 rows only, as a held-out set: the same arrays behind an offset row pointer
    X = api.matrix_from_workload(w)
    held = api.Matrix(1000, w.d, row_ptr=X.row_ptr[5000:], col_idx=X.col_idx, vals=X.vals)
    y = torch.from_numpy(w.y).cuda()
    got = api.wpsgd_objective(held, y[5000:], torch.from_numpy(wvec).cuda(), 1e-3, loss).cpu().numpy()
    rp = w.row_ptr[5000:] - w.row_ptr[5000]
    lo, hi = w.row_ptr[5000], w.row_ptr[6000]
    obj, err = orc.objective(orc.CSR(rp, w.col_idx[lo:hi], w.vals[lo:hi], w.d), w.y[5000:], wvec.astype(np.float64), 1e-3, loss)
    assert got[0] == pytest.approx(obj, rel=1e-11)
    assert abs(got[1] - err) <= 1e-3


def test_objective_rejects_bad_arguments():
    X = api.Matrix(4, 8, dense=torch.zeros((4, 8), dtype=torch.float32, device="cuda"))
    y = torch.ones(4, dtype=torch.float32, device="cuda")
    w = torch.zeros(8, dtype=torch.float32, device="cuda")
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_objective(X, y, w, -1.0, wl.HINGE)
    assert e.value.status == api.INVALID_ARG
    with pytest.raises(api.WpsgdError) as e:
        api.wpsgd_objective(X, y, w, 0.1, wl.HINGE, workspace=torch.empty(256, dtype=torch.uint8, device="cuda")[:16])
    assert e.value.status in (api.INVALID_ARG, api.WORKSPACE_TOO_SMALL)


# ------------------------------------------------------------------ the unbalanced-cluster experiment, small

def test_weighted_average_beats_the_plain_average_on_unbalanced_chains():
    """Section V, "Analog data", at a small size: eight fast chains and two with a fifth of the
    steps, every chain started from the constant vector 4.  The slow chains have contracted less
    towards the optimum, so averaging them in with full weight (plain averaging) must give a
    worse held-out objective than the weights of Eq. 6; with equal step counts the two agree.
    Every number is also checked against the oracle."""
    w = wl.analog_binary(m_train=20000, m_test=4000, d=3000, n_fast=6000)
    eta, lam = 0.05, 0.01                          # (1 - eta*lambda)^6000 = 0.05, ^1200 = 0.55
    mt = w.meta["m_train"]
    X = api.matrix_from_workload(w)
    train = api.Matrix(mt, w.d, row_ptr=X.row_ptr[:mt + 1], col_idx=X.col_idx, vals=X.vals)
    test = api.Matrix(w.m - mt, w.d, row_ptr=X.row_ptr[mt:], col_idx=X.col_idx, vals=X.vals)
    y = torch.from_numpy(w.y).cuda()
    w0 = torch.full((w.d,), float(w.meta["w0"]), dtype=torch.float32, device="cuda")
    W = api.wpsgd_run_chains_from(train, y[:mt], w.n_steps, eta, lam, w.loss, w.seed, w_start=w0)
    a = api.wpsgd_weights(w.n_steps, eta, lam)
    assert a[-1] < 0.02 < 0.1 < a[0]               # the slow chains are almost switched off
    v_wp = api.wpsgd_combine(W, a)
    v_avg = api.wpsgd_combine(W, np.full(w.k, 1.0 / w.k))
    obj_wp, err_wp = api.wpsgd_objective(test, y[mt:], v_wp, lam, w.loss).cpu().numpy()
    obj_avg, err_avg = api.wpsgd_objective(test, y[mt:], v_avg, lam, w.loss).cpu().numpy()
    assert obj_wp < 0.8 * obj_avg
    assert err_wp <= err_avg

    # the same numbers from the oracle
    lo, hi = int(w.row_ptr[0]), int(w.row_ptr[mt])
    Xo_train = orc.CSR(w.row_ptr[:mt + 1], w.col_idx[lo:hi], w.vals[lo:hi], w.d)
    rp = w.row_ptr[mt:] - w.row_ptr[mt]
    Xo_test = orc.CSR(rp, w.col_idx[hi:], w.vals[hi:], w.d)
    Wo, _ = orc.run_chains(Xo_train, w.y[:mt], w.n_steps, eta, lam, w.loss, w.seed, w0_fill=float(w.meta["w0"]),
                           csr_mode=orc.LAZY)
    vo = orc.combine(Wo, orc.weights(w.n_steps, eta, lam))
    assert np.linalg.norm(v_wp.cpu().numpy() - vo) / np.linalg.norm(vo) <= TOL
    o_wp, e_wp = orc.objective(Xo_test, w.y[mt:], v_wp.cpu().numpy().astype(np.float64), lam, w.loss)
    assert obj_wp == pytest.approx(o_wp, rel=1e-11) and abs(err_wp - e_wp) <= 1.0 / (w.m - mt)


# ------------------------------------------------------------------ error paths

def test_run_chains_rejects_bad_arguments():
    w = wl.tiny_hinge(n_steps=(10, 5))
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    for kwargs in [dict(eta=0.0), dict(lam=-1.0), dict(eta=10.0, lam=0.2)]:
        args = dict(eta=w.eta, lam=w.lam)
        args.update(kwargs)
        with pytest.raises(api.WpsgdError) as err:
            api.wpsgd_run_chains(X, y, w.n_steps, args["eta"], args["lam"], w.loss, 0)
        assert err.value.status == api.INVALID_ARG
    with pytest.raises(api.WpsgdError) as err:
        api.wpsgd_run_chains(X, y, [10, -1], w.eta, w.lam, w.loss, 0)
    assert err.value.status == api.INVALID_ARG
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(api.WpsgdError) as err:
        api.wpsgd_run_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, 0, workspace=small)
    assert err.value.status == api.WORKSPACE_TOO_SMALL
    with pytest.raises(api.WpsgdError) as err:
        api.wpsgd_run_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, 0, plan={"threads": 64, "block_steps": 8})
    assert err.value.status == api.UNSUPPORTED
    torch.cuda.synchronize()


# ------------------------------------------------------------------ the five workloads at full size

def test_full_dense_logistic():
    w = wl.dense_logistic()
    W = gpu_chains(w)
    check_against_oracle(w, W, label="dense_logistic full")          # the oracle runs all 64 chains


def test_full_many_chains():
    w = wl.many_chains()
    W = gpu_chains(w)
    check_against_oracle(w, W, label="many_chains full")             # all 2048 chains


def test_full_wide_bf16():
    w = wl.wide_bf16()
    W = gpu_chains(w)
    check_against_oracle(w, W, label="wide_bf16 full")               # all 32 chains and the final model


def test_full_sparse_hinge():
    w = wl.sparse_hinge()
    W = gpu_chains(w)
    # The plain oracle shrinks all 2^20 coordinates at every step, so it recomputes the six
    # shortest chains and the median one.
    by_len = np.argsort(w.n_steps)
    ids = np.array(sorted(set(by_len[:6].tolist()) | {int(by_len[w.k // 2])}))
    check_against_oracle(w, W, chain_ids=ids, label="sparse_hinge full")
    # All 128 chains and the final model against the oracle's scalar-scale mode.
    errs, margin = check_against_oracle(w, W, label="sparse_hinge full, every chain", csr_mode=orc.LAZY)
    assert (margin >= KINK).all(), f"a chain came within {margin.min()} of the hinge kink"
