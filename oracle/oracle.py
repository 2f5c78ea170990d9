"""ctypes front end of the WP-SGD reference oracle (oracle/wpsgd_oracle.c).

TEST INFRASTRUCTURE ONLY.  The product path never imports this module; it is
used by tests/, by the smoke check and by the CPU-baseline leg of the
benchmark.  It shares no code with the HIP library.

All arithmetic happens in the C file; this module only marshals numpy arrays.
`build()` compiles the C file with gcc when the shared object is missing or
older than its source.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "wpsgd_oracle.c")
_LIB = os.path.join(_HERE, "libwpsgd_oracle.so")

HINGE, LOGISTIC = 0, 1
F32, BF16, F64 = 0, 1, 2
PLAIN, LAZY = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-pthread", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


def _p(arr, ctype):
    return None if arr is None else arr.ctypes.data_as(ctypes.POINTER(ctype))


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i64, f64, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        pi64, pf64 = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double)
        pf32, pi32 = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int32)
        pu32 = ctypes.POINTER(ctypes.c_uint32)
        vp = ctypes.c_void_p
        L.oracle_philox4x32_10.argtypes = [pu32, pu32, pu32]
        L.oracle_philox4x32_10.restype = None
        L.oracle_sample_indices.argtypes = [ctypes.c_uint64, i64, i64, i64, i64, pi64]
        L.oracle_shard_indices.argtypes = [ctypes.c_uint64, i64, i64, i64, i64, i64, pi64]
        L.oracle_sgd_dense.argtypes = [vp, i32, i64, i64, pf32, pi64, i64, f64, f64, i32, pf64, pf64]
        L.oracle_sgd_csr.argtypes = [pi64, pi32, pf32, i64, i64, pf32, pi64, i64, f64, f64, i32, i32, pf64, pf64]
        L.oracle_weights_rate.argtypes = [i64, pi64, f64, pf64]
        L.oracle_weights.argtypes = [i64, pi64, f64, f64, pf64]
        L.oracle_benefit_margin.argtypes = [i64, pi64, f64, pf64]
        L.oracle_span_condition.argtypes = [i64, pi64, f64, pf64]
        L.oracle_combine.argtypes = [pf64, pf64, i64, i64, pf64]
        L.oracle_objective.argtypes = [vp, i32, pi64, pi32, pf32, i64, i64, pf32, pf64, f64, i32, pf64, pf64]
        L.oracle_run_chains.argtypes = [vp, i32, pi64, pi32, pf32, i64, i64, pf32, i64, pi64, pi64,
                                        f64, f64, i32, i32, ctypes.c_uint64, f64, i32, pf64, pf64]
        L.oracle_check_triple.argtypes = [f64, f64, f64, f64, f64, f64, pf64]
        L.oracle_delay_sgd_dense.argtypes = [vp, i32, i64, i64, pf32, pi64, i64, f64, f64, i32, i32, i32,
                                             pf64, pi64, pf64]
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c, ctypes.c_uint32), _p(k, ctypes.c_uint32), _p(out, ctypes.c_uint32))
    return out


def shard_indices(seed, chain, k, n0, count, m):
    """Rows node `chain` of k visits at steps n0.. under partition-and-shuffle sampling (Algorithm 1)."""
    out = np.zeros(max(int(count), 0), dtype=np.int64)
    _check(lib().oracle_shard_indices(ctypes.c_uint64(int(seed)), ctypes.c_int64(int(chain)), ctypes.c_int64(int(k)),
                                      ctypes.c_int64(int(n0)), ctypes.c_int64(int(count)), ctypes.c_int64(int(m)),
                                      _p(out, ctypes.c_int64)), "shard_indices")
    return out


def sample_indices(seed, chain, n0, count, m):
    out = np.zeros(max(int(count), 0), dtype=np.int64)
    _check(lib().oracle_sample_indices(int(seed), int(chain), int(n0), int(count), int(m),
                                       _p(out, ctypes.c_int64)), "sample_indices")
    return out


class Dense:
    """Row-major m x d matrix; data is float32, float64, or uint16 holding bfloat16 bits."""

    def __init__(self, data):
        data = np.ascontiguousarray(data)
        assert data.ndim == 2
        self.data = data
        self.m, self.d = data.shape
        self.xtype = {np.dtype(np.float32): F32, np.dtype(np.uint16): BF16,
                      np.dtype(np.float64): F64}[data.dtype]


class CSR:
    """CSR matrix: int64 row_ptr (m+1), int32 col_idx, float32 vals."""

    def __init__(self, row_ptr, col_idx, vals, d):
        self.row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
        self.col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
        self.vals = np.ascontiguousarray(vals, dtype=np.float32)
        self.m = self.row_ptr.size - 1
        self.d = int(d)


def _y32(y):
    return np.ascontiguousarray(y, dtype=np.float32)


def sgd(X, y, idx, eta, lam, loss, w0=None, csr_mode=PLAIN):
    """Run one chain over the explicit visit order idx; returns (w_n, min |1 - y*yhat|)."""
    y = _y32(y)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    w = np.zeros(X.d, dtype=np.float64) if w0 is None else np.array(w0, dtype=np.float64).copy()
    assert w.shape == (X.d,) and y.shape == (X.m,)
    mm = ctypes.c_double(0.0)
    if isinstance(X, Dense):
        rc = lib().oracle_sgd_dense(X.data.ctypes.data, X.xtype, X.m, X.d, _p(y, ctypes.c_float),
                                    _p(idx, ctypes.c_int64), idx.size, float(eta), float(lam),
                                    int(loss), _p(w, ctypes.c_double), ctypes.byref(mm))
    else:
        rc = lib().oracle_sgd_csr(_p(X.row_ptr, ctypes.c_int64), _p(X.col_idx, ctypes.c_int32),
                                  _p(X.vals, ctypes.c_float), X.m, X.d, _p(y, ctypes.c_float),
                                  _p(idx, ctypes.c_int64), idx.size, float(eta), float(lam),
                                  int(loss), int(csr_mode), _p(w, ctypes.c_double), ctypes.byref(mm))
    _check(rc, "sgd")
    return w, mm.value


def weights(n_steps, eta, lam):
    n = np.ascontiguousarray(n_steps, dtype=np.int64)
    a = np.zeros(n.size, dtype=np.float64)
    _check(lib().oracle_weights(n.size, _p(n, ctypes.c_int64), float(eta), float(lam),
                                _p(a, ctypes.c_double)), "weights")
    return a


def weights_rate(n_steps, rate):
    n = np.ascontiguousarray(n_steps, dtype=np.int64)
    a = np.zeros(n.size, dtype=np.float64)
    _check(lib().oracle_weights_rate(n.size, _p(n, ctypes.c_int64), float(rate),
                                     _p(a, ctypes.c_double)), "weights_rate")
    return a


def benefit_margin(n_steps, rate):
    n = np.ascontiguousarray(n_steps, dtype=np.int64)
    out = ctypes.c_double(0.0)
    _check(lib().oracle_benefit_margin(n.size, _p(n, ctypes.c_int64), float(rate),
                                       ctypes.byref(out)), "benefit_margin")
    return out.value


def span_condition(steps_per_span, rate):
    """Left side of the validity condition below Deduction 2 (valid when < 1)."""
    n = np.ascontiguousarray(steps_per_span, dtype=np.int64)
    out = ctypes.c_double(0.0)
    _check(lib().oracle_span_condition(n.size, _p(n, ctypes.c_int64), float(rate),
                                       ctypes.byref(out)), "span_condition")
    return out.value


def combine(W, a):
    W = np.ascontiguousarray(W, dtype=np.float64)
    a = np.ascontiguousarray(a, dtype=np.float64)
    k, d = W.shape
    assert a.shape == (k,)
    v = np.zeros(d, dtype=np.float64)
    _check(lib().oracle_combine(_p(W, ctypes.c_double), _p(a, ctypes.c_double), k, d,
                                _p(v, ctypes.c_double)), "combine")
    return v


def objective(X, y, w, lam, loss):
    """(regularised objective, error rate) of model w on (X, y)."""
    y = _y32(y)
    w = np.ascontiguousarray(w, dtype=np.float64)
    obj, err = ctypes.c_double(0.0), ctypes.c_double(0.0)
    if isinstance(X, Dense):
        rc = lib().oracle_objective(X.data.ctypes.data, X.xtype, None, None, None, X.m, X.d,
                                    _p(y, ctypes.c_float), _p(w, ctypes.c_double), float(lam),
                                    int(loss), ctypes.byref(obj), ctypes.byref(err))
    else:
        rc = lib().oracle_objective(None, 0, _p(X.row_ptr, ctypes.c_int64),
                                    _p(X.col_idx, ctypes.c_int32), _p(X.vals, ctypes.c_float),
                                    X.m, X.d, _p(y, ctypes.c_float), _p(w, ctypes.c_double),
                                    float(lam), int(loss), ctypes.byref(obj), ctypes.byref(err))
    _check(rc, "objective")
    return obj.value, err.value


def run_chains(X, y, n_steps, eta, lam, loss, seed, chain_ids=None, csr_mode=PLAIN,
               w0_fill=0.0, threads=None):
    """Chains of Algorithm 1.  n_steps has one entry per chain of the whole job;
    chain_ids (default: all) selects which of them to compute.  Returns
    (W [len(chain_ids) x d] float64, min_margin [len(chain_ids)])."""
    y = _y32(y)
    n_all = np.ascontiguousarray(n_steps, dtype=np.int64)
    ids = np.arange(n_all.size, dtype=np.int64) if chain_ids is None else \
        np.ascontiguousarray(chain_ids, dtype=np.int64)
    n_sel = np.ascontiguousarray(n_all[ids])
    W = np.zeros((ids.size, X.d), dtype=np.float64)
    mm = np.zeros(ids.size, dtype=np.float64)
    if threads is None:
        threads = min(ids.size, len(os.sched_getaffinity(0)))
    if isinstance(X, Dense):
        args = (X.data.ctypes.data, X.xtype, None, None, None)
    else:
        args = (None, 0, _p(X.row_ptr, ctypes.c_int64), _p(X.col_idx, ctypes.c_int32),
                _p(X.vals, ctypes.c_float))
    rc = lib().oracle_run_chains(*args, X.m, X.d, _p(y, ctypes.c_float), ids.size,
                                 _p(ids, ctypes.c_int64), _p(n_sel, ctypes.c_int64),
                                 float(eta), float(lam), int(loss), int(csr_mode), int(seed),
                                 float(w0_fill), int(threads), _p(W, ctypes.c_double),
                                 _p(mm, ctypes.c_double))
    _check(rc, "run_chains")
    return W, mm


def run_spans(X, y, steps_per_span, n_spans, eta, lam, loss, seed, w0=None, shards=False,
              csr_mode=PLAIN):
    """Periodic weighted averaging (Section III, Deduction 2): n_spans times, chain i takes
    steps_per_span[i] steps from the common vector v, continuing its own visit order, and v
    becomes the Eq. 6 weighted sum of the chains' results.  The steps themselves are sgd(),
    the weights weights(), the sum combine(): nothing else happens here.  Returns v."""
    n = np.ascontiguousarray(steps_per_span, dtype=np.int64)
    k = n.size
    v = np.zeros(X.d, dtype=np.float64) if w0 is None else np.array(w0, dtype=np.float64).copy()
    a = weights(n, eta, lam)
    for s in range(int(n_spans)):
        W = np.zeros((k, X.d), dtype=np.float64)
        for i in range(k):
            first = s * int(n[i])
            idx = shard_indices(seed, i, k, first, int(n[i]), X.m) if shards else \
                sample_indices(seed, i, first, int(n[i]), X.m)
            W[i], _ = sgd(X, y, idx, eta, lam, loss, w0=v, csr_mode=csr_mode)
        v = combine(W, a)
    return v


def check_triple(La, Lb, Lc, pa, pb, rate):
    """Algorithm 4 on one triple of consecutive iterates: projections La, Lb, Lc on the sample and the
    squared perpendicular lengths pa, pb of the two older ones.  Returns (accepted, gap)."""
    gap = ctypes.c_double(0.0)
    ok = lib().oracle_check_triple(float(La), float(Lb), float(Lc), float(pa), float(pb), float(rate),
                                   ctypes.byref(gap))
    return bool(ok), gap.value


def delay_sgd(X, y, idx, eta, lam, loss, tau, w0=None, check=True):
    """One server of Algorithm 3 (delay SGD with the Check function of Algorithm 4) over the explicit
    visit order idx.  Returns (last accepted iterate, number of accepted updates, closest tie)."""
    assert isinstance(X, Dense)
    y = _y32(y)
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    w = np.zeros(X.d, dtype=np.float64) if w0 is None else np.array(w0, dtype=np.float64).copy()
    acc, gap = ctypes.c_int64(0), ctypes.c_double(0.0)
    _check(lib().oracle_delay_sgd_dense(X.data.ctypes.data, X.xtype, X.m, X.d, _p(y, ctypes.c_float),
                                        _p(idx, ctypes.c_int64), idx.size, float(eta), float(lam), int(loss),
                                        int(tau), int(bool(check)), _p(w, ctypes.c_double), ctypes.byref(acc),
                                        ctypes.byref(gap)), "delay_sgd")
    return w, int(acc.value), gap.value


def run_delay_chains(X, y, n_samples, eta, lam, loss, seed, tau, check=True):
    """All servers of Algorithm 3, phase 1: server i consumes n_samples[i] samples of its own stream.
    Returns (W [k x d], accepted [k], closest tie [k])."""
    n = np.ascontiguousarray(n_samples, dtype=np.int64)
    W = np.zeros((n.size, X.d), dtype=np.float64)
    acc = np.zeros(n.size, dtype=np.int64)
    gap = np.zeros(n.size, dtype=np.float64)
    for i in range(n.size):
        W[i], acc[i], gap[i] = delay_sgd(X, y, sample_indices(seed, i, 0, int(n[i]), X.m), eta, lam, loss, tau,
                                         check=check)
    return W, acc, gap


def wpsgd(X, y, n_steps, eta, lam, loss, seed, threads=None):
    """Whole path of Algorithm 1: chains, Eq. 6 weights, weighted sum.  Returns (v, W, a)."""
    W, _ = run_chains(X, y, n_steps, eta, lam, loss, seed, threads=threads)
    a = weights(n_steps, eta, lam)
    return combine(W, a), W, a
