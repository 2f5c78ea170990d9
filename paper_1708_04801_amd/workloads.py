"""Seeded synthetic workloads for the WP-SGD chains.

This module only *generates inputs* (data matrix, labels, per-chain step
counts, hyper-parameters).  It holds none of the method's arithmetic: no SGD
step, no weights, no sample-index stream.  The same arrays are handed to the
GPU library and to the reference oracle.

Five workload families, each with a full-size default and keyword overrides so
the tests can ask for a small instance of the same structure:

  tiny_hinge      dense fp32, hinge,    m=4096     d=64     k=4
  dense_logistic  dense fp32, logistic, m=262144   d=4096   k=64
  sparse_hinge    CSR,        hinge,    m=1000000  d=2^20   k=128  (~80 nnz/row, Zipf columns)
  many_chains     dense fp32, hinge,    m=1048576  d=256    k=2048
  wide_bf16       dense bf16, logistic, m=65536    d=65536  k=32

and one for the delay-SGD servers of Section IV:

  delay_servers   dense fp32, logistic, m=65536    d=4096   k=128  (rows nearly along one direction)

The sparse family stands in for the very wide, very sparse, hinge-loss text-like
data the paper trains on (section V, "Real-world data"); it borrows only the
shape class, none of that data set's records.

Everything is drawn from numpy PCG64 generators spawned from one SeedSequence
per workload, one child per row block, so the result does not depend on the
number of worker threads.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

HINGE, LOGISTIC = 0, 1


@dataclass
class Workload:
    name: str
    loss: int                      # HINGE / LOGISTIC
    eta: float
    lam: float
    seed: int                      # Philox seed of the sample-index stream
    n_steps: np.ndarray            # int64 [k], steps each chain runs
    y: np.ndarray                  # float32 [m], +-1
    m: int
    d: int
    dense: Optional[np.ndarray] = None     # float32 [m,d] or uint16 (bfloat16 bits) [m,d]
    row_ptr: Optional[np.ndarray] = None   # int64 [m+1]
    col_idx: Optional[np.ndarray] = None   # int32 [nnz], strictly ascending within a row
    vals: Optional[np.ndarray] = None      # float32 [nnz]
    meta: dict = field(default_factory=dict)

    @property
    def k(self) -> int:
        return int(self.n_steps.size)

    @property
    def is_csr(self) -> bool:
        return self.dense is None

    @property
    def is_bf16(self) -> bool:
        return self.dense is not None and self.dense.dtype == np.uint16

    def row_bytes(self) -> float:
        """Bytes of one stored sample row (mean over rows for CSR: columns + values)."""
        if self.is_csr:
            return 8.0 * self.vals.size / self.m
        return float(self.d * self.dense.dtype.itemsize)


def _workers() -> int:
    return max(1, min(16, len(os.sched_getaffinity(0))))


def _blocks(m: int, rows_per_block: int):
    return [(lo, min(m, lo + rows_per_block)) for lo in range(0, m, rows_per_block)]


def _run_blocks(fn, blocks, seeds):
    with ThreadPoolExecutor(max_workers=_workers()) as pool:
        return list(pool.map(lambda a: fn(a[0][0], a[0][1], np.random.default_rng(a[1])),
                             zip(blocks, seeds)))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _dense_matrix(m, d, scale, ss, store_bf16, wstar, label_fn):
    """Fill X (m x d) block by block; labels come from label_fn(block_f32, rng)."""
    X = np.empty((m, d), dtype=np.uint16 if store_bf16 else np.float32)
    y = np.empty(m, dtype=np.float32)
    rows = max(1, min(m, (1 << 24) // max(d, 1)))
    blocks = _blocks(m, rows)

    def fill(lo, hi, rng):
        blk = rng.standard_normal((hi - lo, d), dtype=np.float32)
        if scale != 1.0:
            blk *= np.float32(scale)
        if store_bf16:
            bits = f32_to_bf16_bits(blk)
            X[lo:hi] = bits
            blk = bf16_bits_to_f32(bits)      # labels see the stored values
        else:
            X[lo:hi] = blk
        y[lo:hi] = label_fn(blk @ wstar, rng)
        return None

    _run_blocks(fill, blocks, ss.spawn(len(blocks)))
    return X, y


def _sign_labels(noise):
    def fn(score, rng):
        s = score + noise * rng.standard_normal(score.shape[0]) if noise else score
        return np.where(s >= 0, 1.0, -1.0).astype(np.float32)
    return fn


def _logistic_labels(score, rng):
    p = 1.0 / (1.0 + np.exp(-score.astype(np.float64)))
    return np.where(rng.random(score.shape[0]) < p, 1.0, -1.0).astype(np.float32)


def tiny_hinge(m=4096, d=64, n_steps=(1000, 800, 600, 400), data_seed=1001) -> Workload:
    ss = np.random.SeedSequence(data_seed)
    s_w, s_x = ss.spawn(2)
    wstar = (np.random.default_rng(s_w).standard_normal(d) / np.sqrt(d)).astype(np.float32)
    X, y = _dense_matrix(m, d, 1.0, s_x, False, wstar, _sign_labels(0.1))
    return Workload("tiny_hinge", HINGE, 0.01, 1e-3, 0, np.asarray(n_steps, dtype=np.int64),
                    y, m, d, dense=X)


def dense_logistic(m=262144, d=4096, k=64, n_lo=5000, n_hi=20000, data_seed=1002) -> Workload:
    ss = np.random.SeedSequence(data_seed)
    s_w, s_x, s_n = ss.spawn(3)
    wstar = np.random.default_rng(s_w).standard_normal(d).astype(np.float32)
    X, y = _dense_matrix(m, d, 1.0 / np.sqrt(d), s_x, False, wstar, _logistic_labels)
    n = np.random.default_rng(s_n).integers(n_lo, n_hi + 1, size=k).astype(np.int64)
    return Workload("dense_logistic", LOGISTIC, 0.05, 1e-4, 0, n, y, m, d, dense=X)


def many_chains(m=1048576, d=256, k=2048, n_full=2000, data_seed=1004) -> Workload:
    ss = np.random.SeedSequence(data_seed)
    s_w, s_x, s_n = ss.spawn(3)
    wstar = (np.random.default_rng(s_w).standard_normal(d) / np.sqrt(d)).astype(np.float32)
    X, y = _dense_matrix(m, d, 1.0, s_x, False, wstar, _sign_labels(0.1))
    speed = np.random.default_rng(s_n).uniform(0.25, 1.0, size=k)
    n = np.rint(n_full * speed).astype(np.int64)
    return Workload("many_chains", HINGE, 0.01, 1e-3, 0, n, y, m, d, dense=X,
                    meta={"n_full": n_full})


def wide_bf16(m=65536, d=65536, k=32, n_levels=(8000, 4000, 2000, 1000), data_seed=1005) -> Workload:
    ss = np.random.SeedSequence(data_seed)
    s_w, s_x = ss.spawn(2)
    wstar = np.random.default_rng(s_w).standard_normal(d).astype(np.float32)
    X, y = _dense_matrix(m, d, 1.0 / np.sqrt(d), s_x, True, wstar, _logistic_labels)
    reps = -(-k // len(n_levels))
    n = np.repeat(np.asarray(n_levels, dtype=np.int64), reps)[:k]
    return Workload("wide_bf16", LOGISTIC, 0.02, 1e-5, 0, n, y, m, d, dense=X)


def sparse_hinge(m=1_000_000, d=1 << 20, k=128, nnz_mean=80, n_median=10000, n_sigma=0.7,
                 zipf_a=1.1, data_seed=1003) -> Workload:
    """CSR rows: length ~ Poisson(nnz_mean) clipped to [1, 256]; columns are distinct draws
    from Zipf(zipf_a) over ranks 1..d (column = rank - 1, so low columns are hot); values
    lognormal(0, 1); every row scaled to unit L2 norm.  Labels: sign of w*.x with w* 5 % dense."""
    ss = np.random.SeedSequence(data_seed)
    s_w, s_x, s_n = ss.spawn(3)
    rng_w = np.random.default_rng(s_w)
    wstar = np.zeros(d, dtype=np.float64)
    support = rng_w.choice(d, size=max(1, d // 20), replace=False)
    wstar[support] = rng_w.standard_normal(support.size)

    cdf = np.cumsum(np.arange(1, d + 1, dtype=np.float64) ** (-zipf_a))
    cdf /= cdf[-1]
    max_len = 256
    cand = 2 * min(max_len, int(nnz_mean + 6 * np.sqrt(nnz_mean))) + 16   # draws per row
    blocks = _blocks(m, 32768)

    def fill(lo, hi, rng):
        r = hi - lo
        want = np.clip(rng.poisson(nnz_mean, size=r), 1, max_len)
        cols = np.searchsorted(cdf, rng.random((r, cand)), side="left").astype(np.int64)
        np.minimum(cols, d - 1, out=cols)
        cols.sort(axis=1)
        dup = np.zeros((r, cand), dtype=bool)
        dup[:, 1:] = cols[:, 1:] == cols[:, :-1]
        prio = rng.random((r, cand))
        prio[dup] = 2.0                                   # duplicates are never kept
        rank = prio.argsort(axis=1).argsort(axis=1)       # position of each draw in priority order
        n_unique = cand - dup.sum(axis=1)
        keep = rank < np.minimum(want, n_unique)[:, None]
        lens = keep.sum(axis=1)
        c = cols[keep].astype(np.int32)                   # row-major order keeps columns ascending
        v = rng.lognormal(0.0, 1.0, size=c.size)
        ptr = np.concatenate(([0], np.cumsum(lens)))
        sq = np.add.reduceat(v * v, ptr[:-1])
        v /= np.repeat(np.sqrt(sq), lens)
        v32 = v.astype(np.float32)
        score = np.add.reduceat(v32.astype(np.float64) * wstar[c], ptr[:-1])
        lab = np.where(score >= 0, 1.0, -1.0).astype(np.float32)
        return lens, c, v32, lab

    parts = _run_blocks(fill, blocks, s_x.spawn(len(blocks)))
    lens = np.concatenate([p[0] for p in parts])
    row_ptr = np.zeros(m + 1, dtype=np.int64)
    np.cumsum(lens, out=row_ptr[1:])
    col_idx = np.concatenate([p[1] for p in parts])
    vals = np.concatenate([p[2] for p in parts])
    y = np.concatenate([p[3] for p in parts])
    n = np.rint(np.random.default_rng(s_n).lognormal(np.log(n_median), n_sigma, size=k)).astype(np.int64)
    return Workload("sparse_hinge", HINGE, 0.1, 1e-5, 0, n, y, m, d,
                    row_ptr=row_ptr, col_idx=col_idx, vals=vals)


def analog_binary(m_train=460_000, m_test=40_000, d=100_000, n_fast=100_000, fast=8, slow=2, slow_share=0.2,
                  data_seed=1006) -> Workload:
    """The fully specified synthetic data of the paper's "Analog data" experiment (section V):
    rows with 5 to 10 binary features at random positions, scaled to unit length; the label is
    the sign of sum_i x_i * (i % 4) * (-1)^i over the 1-based feature index i (+1 where the paper
    writes label 1, -1 where it writes 0).  The first m_train rows are for training, the rest
    for testing.  `fast` chains run n_fast steps, `slow` chains slow_share of that (the paper's
    unbalanced cluster: eight nodes with five times the data of the other two).  eta, lambda as
    in the paper; meta carries its start value 4 and its fitted contraction rate 0.99999."""
    m = m_train + m_test
    rng = np.random.default_rng(data_seed)
    lens = rng.integers(5, 11, size=m)
    row_ptr = np.concatenate(([0], np.cumsum(lens))).astype(np.int64)
    # ten distinct positions per row (rejection on the rare repeats), the first lens[r] are kept
    cand = rng.integers(0, d, size=(m, 10))
    while True:
        srt = np.sort(cand, axis=1)
        bad = (srt[:, 1:] == srt[:, :-1]).any(axis=1)
        if not bad.any():
            break
        cand[bad] = rng.integers(0, d, size=(int(bad.sum()), 10))
    keep = np.arange(10)[None, :] < lens[:, None]
    cols = np.where(keep, cand, d)                     # dropped slots sort to the end
    cols.sort(axis=1)
    col_idx = cols[cols < d].astype(np.int32)           # row-major: ascending inside every row
    i1 = col_idx.astype(np.int64) + 1                  # the paper counts features from 1
    score = np.add.reduceat((i1 % 4) * np.where(i1 % 2 == 0, 1.0, -1.0), row_ptr[:-1])
    vals = np.repeat(1.0 / np.sqrt(lens), lens).astype(np.float32)
    y = np.where(score > 0, 1.0, -1.0).astype(np.float32)
    n = np.array([n_fast] * fast + [int(round(n_fast * slow_share))] * slow, dtype=np.int64)
    return Workload("analog_binary", HINGE, 1e-4, 0.01, 0, n, y, m, d, row_ptr=row_ptr, col_idx=col_idx, vals=vals,
                    meta={"m_train": m_train, "m_test": m_test, "w0": 4.0, "rate": 0.99999})


def delay_servers(m=65536, d=4096, k=128, n_lo=2000, n_hi=8000, tau=2, loss=LOGISTIC, spread=0.01, bf16=False,
                  data_seed=1006) -> Workload:
    """Input for the delay-SGD servers (Section IV).  On unstructured rows the acceptance test of that
    section throws away nearly every sample after the first, so the rows here lie close to one
    direction u: x_j = y_j * s_j * u + noise, s_j uniform in [0.6, 1], |u| = 1, noise of total length
    about `spread`.  Successive projections then move the same way and servers make tens of updates.
    meta: the delay tau and a common non-zero start vector (float32)."""
    ss = np.random.SeedSequence(data_seed)
    s_u, s_x, s_n, s_w = ss.spawn(4)
    u = np.random.default_rng(s_u).standard_normal(d)
    u = (u / np.linalg.norm(u)).astype(np.float32)
    X = np.empty((m, d), dtype=np.uint16 if bf16 else np.float32)
    y = np.empty(m, dtype=np.float32)
    blocks = _blocks(m, max(1, min(m, (1 << 24) // max(d, 1))))

    def fill(lo, hi, rng):
        lab = np.where(rng.random(hi - lo) < 0.5, 1.0, -1.0).astype(np.float32)
        length = (0.6 + 0.4 * rng.random(hi - lo)).astype(np.float32)
        blk = rng.standard_normal((hi - lo, d), dtype=np.float32)
        blk *= np.float32(spread / np.sqrt(d))
        blk += np.outer(lab * length, u)
        X[lo:hi] = f32_to_bf16_bits(blk) if bf16 else blk
        y[lo:hi] = lab
        return None

    _run_blocks(fill, blocks, s_x.spawn(len(blocks)))
    n = np.random.default_rng(s_n).integers(n_lo, n_hi + 1, size=k).astype(np.int64)
    w_start = (np.random.default_rng(s_w).standard_normal(d) * (1.0 / np.sqrt(d))).astype(np.float32)
    return Workload("delay_servers", loss, 0.5, 0.25, 0, n, y, m, d, dense=X, meta={"tau": tau, "w_start": w_start})


FULL = {
    "tiny_hinge": tiny_hinge,
    "dense_logistic": dense_logistic,
    "sparse_hinge": sparse_hinge,
    "many_chains": many_chains,
    "wide_bf16": wide_bf16,
}
