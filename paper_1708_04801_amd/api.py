"""ctypes binding of libwpsgd.so: same names as the C ABI in include/wpsgd.h.

Argument marshalling only -- every step of the path runs in the HIP library.  PyTorch is
used for device memory (tensors) and for the current HIP stream; nothing here computes.
There is no CPU fallback: if the library is missing or cannot be loaded, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libwpsgd.so")

HINGE, LOGISTIC = 0, 1
SAMPLE_STREAM, SAMPLE_SHARDS = 0, 1
F32, BF16 = 0, 1
OK, INVALID_ARG, HIP_ERROR, WORKSPACE_TOO_SMALL, UNSUPPORTED, INCOMPLETE = 0, -1, -2, -3, -4, -5

EXPORTS = [
    "wpsgd_run_chains_workspace", "wpsgd_run_chains", "wpsgd_weights", "wpsgd_weights_rate",
    "wpsgd_benefit_margin", "wpsgd_combine_workspace", "wpsgd_combine", "wpsgd_sample_indices",
    "wpsgd_sample_indices_device", "wpsgd_strerror", "wpsgd_last_hip_error", "wpsgd_describe_plan",
    "wpsgd_stream_rows", "wpsgd_objective_workspace", "wpsgd_objective",
    "wpsgd_run_chains_from", "wpsgd_shard_indices", "wpsgd_shard_indices_device",
    "wpsgd_run_spans_workspace", "wpsgd_run_spans", "wpsgd_span_condition", "wpsgd_objective_static",
    "wpsgd_chains_status", "wpsgd_run_delay_chains_workspace", "wpsgd_run_delay_chains",
]


class _CMatrix(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("d", ctypes.c_int64), ("dense", ctypes.c_void_p),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int), ("row_ptr", ctypes.c_void_p),
                ("col_idx", ctypes.c_void_p), ("vals", ctypes.c_void_p)]


class _CPlan(ctypes.Structure):
    _fields_ = [("threads", ctypes.c_int), ("block_steps", ctypes.c_int),
                ("prefetch", ctypes.c_int), ("state_in_hbm", ctypes.c_int),
                ("rows", ctypes.c_int), ("helpers", ctypes.c_int), ("slices", ctypes.c_int),
                ("slice_wait_us", ctypes.c_int)]


class WpsgdError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = load().wpsgd_strerror(status).decode()
        if status == HIP_ERROR:
            msg += f" [hipError {load().wpsgd_last_hip_error()}]"
        super().__init__(f"{what}: {msg} (status {status})")


_lib = None


def load():
    """Loads libwpsgd.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1708_04801_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    i64, f64, ci, u64, vp, sz = (ctypes.c_int64, ctypes.c_double, ctypes.c_int, ctypes.c_uint64,
                                 ctypes.c_void_p, ctypes.c_size_t)
    pm, pp = ctypes.POINTER(_CMatrix), ctypes.POINTER(_CPlan)
    L.wpsgd_run_chains_workspace.argtypes = [pm, ci, ci, pp]
    L.wpsgd_run_chains_workspace.restype = sz
    L.wpsgd_run_chains.argtypes = [pm, vp, ci, vp, f64, f64, ci, u64, vp, vp, sz, pp, vp]
    L.wpsgd_run_chains_from.argtypes = [pm, vp, ci, vp, f64, f64, ci, u64, ci, vp, vp, vp, vp, sz, pp, vp]
    L.wpsgd_chains_status.argtypes = [vp, vp]
    L.wpsgd_run_delay_chains_workspace.argtypes = [pm, ci, ci]
    L.wpsgd_run_delay_chains_workspace.restype = sz
    L.wpsgd_run_delay_chains.argtypes = [pm, vp, ci, vp, f64, f64, ci, u64, ci, ci, vp, vp, vp, vp, sz, vp]
    L.wpsgd_run_spans_workspace.argtypes = [pm, ci, ci, pp]
    L.wpsgd_run_spans_workspace.restype = sz
    L.wpsgd_run_spans.argtypes = [pm, vp, ci, vp, i64, f64, f64, ci, u64, ci, vp, vp, vp, sz, pp, vp]
    L.wpsgd_span_condition.argtypes = [ci, vp, f64, vp]
    L.wpsgd_shard_indices.argtypes = [u64, ci, ci, i64, i64, i64, vp]
    L.wpsgd_shard_indices_device.argtypes = [u64, ci, ci, i64, i64, i64, vp, vp]
    L.wpsgd_weights.argtypes = [ci, vp, f64, f64, vp]
    L.wpsgd_weights_rate.argtypes = [ci, vp, f64, vp]
    L.wpsgd_benefit_margin.argtypes = [ci, vp, f64, vp]
    L.wpsgd_combine_workspace.argtypes = [ci, i64]
    L.wpsgd_combine_workspace.restype = sz
    L.wpsgd_combine.argtypes = [vp, vp, ci, i64, vp, vp, sz, vp]
    L.wpsgd_sample_indices.argtypes = [u64, ci, i64, i64, i64, vp]
    L.wpsgd_sample_indices_device.argtypes = [u64, ci, i64, i64, i64, vp, vp]
    L.wpsgd_strerror.argtypes = [ci]
    L.wpsgd_strerror.restype = ctypes.c_char_p
    L.wpsgd_last_hip_error.argtypes = []
    L.wpsgd_describe_plan.argtypes = [pm, ci, ci, pp, ctypes.c_char_p, sz]
    L.wpsgd_stream_rows.argtypes = [pm, ci, i64, u64, vp, vp]
    L.wpsgd_objective_workspace.argtypes = [pm]
    L.wpsgd_objective_workspace.restype = sz
    L.wpsgd_objective.argtypes = [pm, vp, vp, f64, ci, vp, vp, sz, vp]
    L.wpsgd_objective_static.argtypes = [pm, vp, vp, f64, ci, vp, vp]
    _lib = L
    return L


@dataclass
class Matrix:
    """Device-resident data set.  dense: float32 [m,d] tensor, or int16/uint16/bfloat16 [m,d]
    holding bfloat16 values; or CSR with int64 row_ptr, int32 col_idx, float32 vals."""
    m: int
    d: int
    dense: Optional[torch.Tensor] = None
    row_ptr: Optional[torch.Tensor] = None
    col_idx: Optional[torch.Tensor] = None
    vals: Optional[torch.Tensor] = None

    def c_struct(self) -> _CMatrix:
        c = _CMatrix()
        c.m, c.d = int(self.m), int(self.d)
        if self.dense is not None:
            t = self.dense
            assert t.is_cuda and t.dim() == 2 and t.stride(1) == 1
            c.dense = t.data_ptr()
            c.ld = t.stride(0)
            c.dtype = F32 if t.dtype == torch.float32 else BF16
            assert t.dtype in (torch.float32, torch.bfloat16, torch.int16, torch.uint16)
        else:
            assert self.row_ptr.dtype == torch.int64 and self.col_idx.dtype == torch.int32
            assert self.vals.dtype == torch.float32 and self.row_ptr.is_cuda
            c.row_ptr, c.col_idx, c.vals = (self.row_ptr.data_ptr(), self.col_idx.data_ptr(),
                                            self.vals.data_ptr())
        return c


def matrix_from_workload(w, device="cuda") -> Matrix:
    """Uploads a generated workload's data set to the GPU."""
    if w.dense is not None:
        host = torch.from_numpy(w.dense.view(np.int16) if w.dense.dtype == np.uint16 else w.dense)
        dev = host.to(device)
        if w.dense.dtype == np.uint16:
            dev = dev.view(torch.bfloat16)
        return Matrix(w.m, w.d, dense=dev)
    return Matrix(w.m, w.d, row_ptr=torch.from_numpy(w.row_ptr).to(device),
                  col_idx=torch.from_numpy(w.col_idx).to(device),
                  vals=torch.from_numpy(w.vals).to(device))


def _plan(plan):
    if plan is None:
        return None
    p = _CPlan()
    p.threads = int(plan.get("threads", 0))
    p.block_steps = int(plan.get("block_steps", 0))
    p.prefetch = int(plan.get("prefetch", 0))
    p.state_in_hbm = int(plan.get("state_in_hbm", 0))
    p.rows = int(plan.get("rows", 0))
    p.helpers = int(plan.get("helpers", 0))
    p.slices = int(plan.get("slices", 0))
    p.slice_wait_us = int(plan.get("slice_wait_us", 0))
    return ctypes.byref(p)


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _steps(n_steps):
    return np.ascontiguousarray(np.asarray(n_steps), dtype=np.int64)


def _workspace(nbytes, device, stream=None):
    """A temporary workspace for one call.  It is allocated on torch's current stream; when the call's
    work is queued on another stream the caching allocator is told so, or it could hand the block to
    later current-stream work while that stream still uses it."""
    t = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    if stream is not None:
        with torch.cuda.device(t.device):
            t.record_stream(stream if isinstance(stream, torch.cuda.Stream) else torch.cuda.ExternalStream(int(stream)))
    return t


def wpsgd_describe_plan(X: Matrix, k, loss, plan=None) -> str:
    buf = ctypes.create_string_buffer(256)
    cm = X.c_struct()
    rc = load().wpsgd_describe_plan(ctypes.byref(cm), int(k), int(loss), _plan(plan), buf, 256)
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_describe_plan")
    return buf.value.decode()


def wpsgd_run_chains_workspace(X: Matrix, k, loss, plan=None) -> int:
    cm = X.c_struct()
    return int(load().wpsgd_run_chains_workspace(ctypes.byref(cm), int(k), int(loss), _plan(plan)))


def wpsgd_run_chains(X: Matrix, y: torch.Tensor, n_steps, eta, lam, loss, seed,
                     W: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     plan=None, stream=None) -> torch.Tensor:
    """Runs the k chains; returns W (k x d float32 on the GPU).  Asynchronous on the stream."""
    n = _steps(n_steps)
    k = int(n.size)
    dev = y.device
    assert y.is_cuda and y.dtype == torch.float32 and y.numel() == X.m
    if W is None:
        W = torch.empty((k, X.d), dtype=torch.float32, device=dev)
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and W.shape == (k, X.d)
    cm = X.c_struct()
    pl = _plan(plan)
    if workspace is None:
        need = load().wpsgd_run_chains_workspace(ctypes.byref(cm), k, int(loss), pl)
        workspace = _workspace(need, dev, stream)
    rc = load().wpsgd_run_chains(ctypes.byref(cm), y.data_ptr(), k, n.ctypes.data, float(eta),
                                 float(lam), int(loss), int(seed), W.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), pl, _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_run_chains")
    return W


def wpsgd_chains_status(workspace: torch.Tensor, stream=None) -> int:
    """OK, or INCOMPLETE when chains of the last call on this workspace gave up (waits for the stream)."""
    rc = load().wpsgd_chains_status(workspace.data_ptr(), _stream(stream))
    if rc not in (OK, INCOMPLETE):
        raise WpsgdError(rc, "wpsgd_chains_status")
    return rc


def wpsgd_run_chains_from(X: Matrix, y: torch.Tensor, n_steps, eta, lam, loss, seed,
                          w_start: Optional[torch.Tensor] = None, step_offsets=None, sampling=0,
                          W: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                          plan=None, stream=None) -> torch.Tensor:
    """wpsgd_run_chains from a common start vector (d float32 on the GPU, or None for zero) and
    from per-chain positions in the sample streams (k integers, or None for zero)."""
    n = _steps(n_steps)
    k = int(n.size)
    dev = y.device
    assert y.is_cuda and y.dtype == torch.float32 and y.numel() == X.m
    if w_start is not None:
        assert w_start.is_cuda and w_start.dtype == torch.float32 and w_start.is_contiguous() and w_start.numel() == X.d
    off = None
    if step_offsets is not None:
        off = _steps(step_offsets)
        assert off.size == k
    if W is None:
        W = torch.empty((k, X.d), dtype=torch.float32, device=dev)
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and W.shape == (k, X.d)
    cm = X.c_struct()
    pl = _plan(plan)
    if workspace is None:
        need = load().wpsgd_run_chains_workspace(ctypes.byref(cm), k, int(loss), pl)
        workspace = _workspace(need, dev, stream)
    rc = load().wpsgd_run_chains_from(ctypes.byref(cm), y.data_ptr(), k, n.ctypes.data, float(eta),
                                      float(lam), int(loss), int(seed), int(sampling),
                                      w_start.data_ptr() if w_start is not None else None,
                                      off.ctypes.data if off is not None else None, W.data_ptr(),
                                      workspace.data_ptr(), workspace.numel(), pl, _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_run_chains_from")
    return W


def wpsgd_run_delay_chains_workspace(X: Matrix, k, tau) -> int:
    cm = X.c_struct()
    return int(load().wpsgd_run_delay_chains_workspace(ctypes.byref(cm), int(k), int(tau)))


def wpsgd_run_delay_chains(X: Matrix, y: torch.Tensor, n_samples, eta, lam, loss, seed, tau, check=True,
                           w_start: Optional[torch.Tensor] = None, W: Optional[torch.Tensor] = None,
                           accepted: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           stream=None):
    """Phase 1 of delay SGD under the Check function: k servers, server i fed n_samples[i] samples.
    Returns (W, accepted): k x d float32 and k int64, both on the GPU."""
    n = _steps(n_samples)
    k = int(n.size)
    dev = y.device
    assert y.is_cuda and y.dtype == torch.float32 and y.numel() == X.m
    if w_start is not None:
        assert w_start.is_cuda and w_start.dtype == torch.float32 and w_start.is_contiguous() and w_start.numel() == X.d
    if W is None:
        W = torch.empty((k, X.d), dtype=torch.float32, device=dev)
    if accepted is None:
        accepted = torch.empty(k, dtype=torch.int64, device=dev)
    assert W.is_cuda and W.dtype == torch.float32 and W.is_contiguous() and W.shape == (k, X.d)
    assert accepted.is_cuda and accepted.dtype == torch.int64 and accepted.is_contiguous() and accepted.numel() == k
    cm = X.c_struct()
    if workspace is None:
        need = load().wpsgd_run_delay_chains_workspace(ctypes.byref(cm), k, int(tau))
        workspace = _workspace(max(int(need), 256), dev, stream)
    rc = load().wpsgd_run_delay_chains(ctypes.byref(cm), y.data_ptr(), k, n.ctypes.data, float(eta), float(lam),
                                       int(loss), int(seed), int(tau), int(bool(check)),
                                       w_start.data_ptr() if w_start is not None else None, W.data_ptr(),
                                       accepted.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_run_delay_chains")
    return W, accepted


def wpsgd_run_spans_workspace(X: Matrix, k, loss, plan=None) -> int:
    cm = X.c_struct()
    return int(load().wpsgd_run_spans_workspace(ctypes.byref(cm), int(k), int(loss), _plan(plan)))


def wpsgd_run_spans(X: Matrix, y: torch.Tensor, steps_per_span, n_spans, eta, lam, loss, seed,
                    w_start: Optional[torch.Tensor] = None, sampling=0, w_out: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, plan=None, stream=None) -> torch.Tensor:
    """Periodic weighted averaging: n_spans times, chains of steps_per_span steps from the common
    vector, then the Eq. 6 weighted sum.  Returns the vector after the last span (d float32)."""
    n = _steps(steps_per_span)
    k = int(n.size)
    dev = y.device
    assert y.is_cuda and y.dtype == torch.float32 and y.numel() == X.m
    if w_start is not None:
        assert w_start.is_cuda and w_start.dtype == torch.float32 and w_start.is_contiguous() and w_start.numel() == X.d
    if w_out is None:
        w_out = torch.empty(X.d, dtype=torch.float32, device=dev)
    assert w_out.is_cuda and w_out.dtype == torch.float32 and w_out.is_contiguous() and w_out.numel() == X.d
    cm = X.c_struct()
    pl = _plan(plan)
    if workspace is None:
        need = load().wpsgd_run_spans_workspace(ctypes.byref(cm), k, int(loss), pl)
        workspace = _workspace(need, dev, stream)
    rc = load().wpsgd_run_spans(ctypes.byref(cm), y.data_ptr(), k, n.ctypes.data, int(n_spans), float(eta),
                                float(lam), int(loss), int(seed), int(sampling),
                                w_start.data_ptr() if w_start is not None else None, w_out.data_ptr(),
                                workspace.data_ptr(), workspace.numel(), pl, _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_run_spans")
    return w_out


def wpsgd_span_condition(steps_per_span, rate) -> float:
    n = _steps(steps_per_span)
    out = ctypes.c_double(0.0)
    rc = load().wpsgd_span_condition(int(n.size), n.ctypes.data, float(rate), ctypes.addressof(out))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_span_condition")
    return out.value


def wpsgd_weights(n_steps, eta, lam) -> np.ndarray:
    n = _steps(n_steps)
    a = np.zeros(n.size, dtype=np.float64)
    rc = load().wpsgd_weights(int(n.size), n.ctypes.data, float(eta), float(lam), a.ctypes.data)
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_weights")
    return a


def wpsgd_weights_rate(n_steps, rate) -> np.ndarray:
    n = _steps(n_steps)
    a = np.zeros(n.size, dtype=np.float64)
    rc = load().wpsgd_weights_rate(int(n.size), n.ctypes.data, float(rate), a.ctypes.data)
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_weights_rate")
    return a


def wpsgd_benefit_margin(n_steps, rate) -> float:
    n = _steps(n_steps)
    out = ctypes.c_double(0.0)
    rc = load().wpsgd_benefit_margin(int(n.size), n.ctypes.data, float(rate),
                                     ctypes.addressof(out))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_benefit_margin")
    return out.value


def wpsgd_combine_workspace(k, d) -> int:
    return int(load().wpsgd_combine_workspace(int(k), int(d)))


def wpsgd_combine(W: torch.Tensor, a, w_out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """w_out = sum_i a[i] * W[i,:]; returns w_out (d float32 on the GPU)."""
    assert W.is_cuda and W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous()
    k, d = W.shape
    a = np.ascontiguousarray(np.asarray(a), dtype=np.float64)
    assert a.shape == (k,)
    if w_out is None:
        w_out = torch.empty(d, dtype=torch.float32, device=W.device)
    if workspace is None:
        workspace = _workspace(wpsgd_combine_workspace(k, d), W.device, stream)
    rc = load().wpsgd_combine(W.data_ptr(), a.ctypes.data, k, d, w_out.data_ptr(),
                              workspace.data_ptr(), workspace.numel(), _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_combine")
    return w_out


def wpsgd_objective_workspace(X: Matrix) -> int:
    cm = X.c_struct()
    return int(load().wpsgd_objective_workspace(ctypes.byref(cm)))


def wpsgd_objective(X: Matrix, y: torch.Tensor, w: torch.Tensor, lam, loss, out: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Returns a 2-element float64 GPU tensor: [regularised objective, error rate] of model w on (X, y)."""
    assert y.is_cuda and y.dtype == torch.float32 and y.numel() == X.m
    assert w.is_cuda and w.dtype == torch.float32 and w.numel() == X.d and w.is_contiguous()
    cm = X.c_struct()
    if out is None:
        out = torch.empty(2, dtype=torch.float64, device=y.device)
    if workspace is None:
        workspace = _workspace(wpsgd_objective_workspace(X), y.device, stream)
    rc = load().wpsgd_objective(ctypes.byref(cm), y.data_ptr(), w.data_ptr(), float(lam), int(loss), out.data_ptr(),
                                workspace.data_ptr(), workspace.numel(), _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_objective")
    return out


def wpsgd_objective_static(X: Matrix, y: torch.Tensor, w: torch.Tensor, lam, loss, out: torch.Tensor,
                           stream=None) -> torch.Tensor:
    """wpsgd_objective without a workspace: the library's own static device area holds the partial
    sums and the call allocates nothing (`out`, two float64 on the GPU, comes from the caller)."""
    assert y.is_cuda and y.dtype == torch.float32 and y.numel() == X.m
    assert w.is_cuda and w.dtype == torch.float32 and w.numel() == X.d and w.is_contiguous()
    assert out.is_cuda and out.dtype == torch.float64 and out.numel() == 2
    cm = X.c_struct()
    rc = load().wpsgd_objective_static(ctypes.byref(cm), y.data_ptr(), w.data_ptr(), float(lam), int(loss),
                                       out.data_ptr(), _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_objective_static")
    return out


def wpsgd_sample_indices(seed, chain, n0, count, m) -> np.ndarray:
    out = np.zeros(max(int(count), 0), dtype=np.int64)
    rc = load().wpsgd_sample_indices(int(seed), int(chain), int(n0), int(count), int(m),
                                     out.ctypes.data)
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_sample_indices")
    return out


def wpsgd_shard_indices(seed, chain, k, n0, count, m) -> np.ndarray:
    out = np.zeros(max(int(count), 0), dtype=np.int64)
    rc = load().wpsgd_shard_indices(int(seed), int(chain), int(k), int(n0), int(count), int(m), out.ctypes.data)
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_shard_indices")
    return out


def wpsgd_shard_indices_device(seed, chain, k, n0, count, m, device="cuda", stream=None) -> torch.Tensor:
    out = torch.empty(max(int(count), 0), dtype=torch.int64, device=device)
    rc = load().wpsgd_shard_indices_device(int(seed), int(chain), int(k), int(n0), int(count), int(m),
                                           out.data_ptr(), _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_shard_indices_device")
    return out


def wpsgd_sample_indices_device(seed, chain, n0, count, m, device="cuda", stream=None) -> torch.Tensor:
    out = torch.empty(max(int(count), 0), dtype=torch.int64, device=device)
    rc = load().wpsgd_sample_indices_device(int(seed), int(chain), int(n0), int(count), int(m),
                                            out.data_ptr(), _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_sample_indices_device")
    return out


def wpsgd_stream_rows(X: Matrix, groups, rows_per_group, seed=0, stream=None) -> torch.Tensor:
    """Streaming ceiling probe; returns the sink tensor (asynchronous, time it with events)."""
    sink = torch.empty(int(groups) * 256, dtype=torch.float32, device=X.dense.device)
    cm = X.c_struct()
    rc = load().wpsgd_stream_rows(ctypes.byref(cm), int(groups), int(rows_per_group), int(seed),
                                  sink.data_ptr(), _stream(stream))
    if rc != OK:
        raise WpsgdError(rc, "wpsgd_stream_rows")
    return sink
