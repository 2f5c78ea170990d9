#!/usr/bin/env python3
"""Benchmark of the WP-SGD hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic workload that is already resident
in HBM: k SGD chains (wpsgd_run_chains), the weights of Eq. 6 (wpsgd_weights) and the weighted
model average (wpsgd_combine).  The metric is SGD sample-updates per second over all chains.

Prints ONE JSON line.  Besides the throughput it carries
  roofline      achieved algorithmic HBM bandwidth of the chain kernel (bytes a sample-update must
                move x sample-updates per launch / mean launch duration from HIP events recorded
                on the launch stream inside the timed region) against the 8 TB/s peak;
  cpu_baseline  the fp64 CPU oracle timed on this machine's host cores on the same workload.

--workload delay_servers measures the servers of Section IV (Algorithm 3 under the Check function of
Algorithm 4) instead: see bench_delay_servers.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def kernel_source_digest() -> str:
    """Digest of the kernel sources; counter-measured traffic is only quoted for the sources it
    was measured on."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1708_04801_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as fh:
            h.update(name.encode())
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str):
    """HBM bytes per chain-kernel launch from the committed counter summary, or None when the
    kernels have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as fh:
        rec = json.load(fh).get(workload)
    if not rec or rec.get("kernel_source_digest") != kernel_source_digest():
        return None
    return rec.get("hbm_bytes_per_launch")


def bench_delay_servers(args, torch, api, wl) -> int:
    """The servers of Section IV (Algorithm 3): one step is phase 1 (wpsgd_run_delay_chains: every server
    consumes its samples, under the Check function of Algorithm 4 unless --no-check) and phase 2 (the
    weights of Eq. 8 on the servers' accepted updates, wpsgd_weights_rate, and wpsgd_combine).  The
    metric counts samples consumed; a sample's algorithmic traffic is its row and its label."""
    t_gen = time.time()
    w = wl.delay_servers()
    t_gen = time.time() - t_gen
    tau, check = int(w.meta["tau"]), not args.no_check
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    k, d = w.k, w.d
    w_start = torch.from_numpy(w.meta["w_start"]).cuda()
    W = torch.empty((k, d), dtype=torch.float32, device="cuda")
    accepted = torch.empty(k, dtype=torch.int64, device="cuda")
    v = torch.empty(d, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(256, api.wpsgd_run_delay_chains_workspace(X, k, tau)), dtype=torch.uint8, device="cuda")
    ws_comb = torch.empty(max(256, api.wpsgd_combine_workspace(k, d)), dtype=torch.uint8, device="cuda")
    rate = 1.0 - w.eta * w.lam

    def step(ev=None):
        if ev is not None:
            ev[0].record()
        api.wpsgd_run_delay_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed, tau, check=check, w_start=w_start,
                                   W=W, accepted=accepted, workspace=ws)
        if ev is not None:
            ev[1].record()
        a = api.wpsgd_weights_rate(accepted.cpu().numpy(), rate)
        api.wpsgd_combine(W, a, w_out=v, workspace=ws_comb)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    samples = int(w.n_steps.sum())
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernel_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    bytes_per_sample = w.row_bytes() + 4
    achieved = bytes_per_sample * samples / (kernel_ms * 1e-3) / 1e9
    acc = accepted.cpu().numpy()
    out = {
        "metric": "samples/sec consumed by delay-SGD servers (all servers)",
        "value": samples / (ms_per_step * 1e-3),
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "delay_servers", "m": w.m, "d": d, "k": k, "tau": tau, "check": check,
                   "samples_per_step": samples, "storage": "f32",
                   "loss": "hinge" if w.loss == wl.HINGE else "logistic",
                   "accepted_updates_min_mean_max": [int(acc.min()), float(acc.mean()), int(acc.max())]},
        "roofline": {"bound": "hbm", "kernel": "delay_server_kernel (wpsgd_run_delay_chains)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("delay_servers") if check else None,
                     "bytes_per_sample": bytes_per_sample, "kernel_ms": kernel_ms,
                     "most_samples_one_server": int(w.n_steps.max()),
                     "us_per_sample_busiest_server": kernel_ms * 1e3 / max(1, int(w.n_steps.max()))},
        "data_generation_s": t_gen,
    }
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        servers = min(k, 32)
        tc = time.perf_counter()
        Wo = np.zeros((servers, d))
        acc_o = np.zeros(servers, dtype=np.int64)
        for i in range(servers):
            idx = orc.sample_indices(w.seed, i, 0, int(w.n_steps[i]), w.m)
            Wo[i], acc_o[i], _ = orc.delay_sgd(orc.Dense(w.dense), w.y, idx, w.eta, w.lam, w.loss, tau,
                                               w0=w.meta["w_start"].astype(np.float64), check=check)
        tc = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": float(w.n_steps[:servers].sum()) / tc, "unit": "samples/s", "cores": 1,
                               "kind": "oracle", "sample": f"the first {servers} servers in full", "seconds": tc}
        Wg = W[:servers].cpu().numpy().astype(np.float64)
        out["parity_rel_l2"] = float(np.linalg.norm(Wg - Wo) / max(np.linalg.norm(Wo), 1e-300))
        out["parity_accepted_equal"] = bool(np.array_equal(acc[:servers], acc_o))
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="dense_logistic",
                    choices=["tiny_hinge", "dense_logistic", "sparse_hinge", "many_chains", "wide_bf16",
                             "delay_servers"])
    ap.add_argument("--no-check", action="store_true",
                    help="delay_servers: plain delay SGD, every candidate kept (default: under the Check function)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--threads", type=int, default=0)
    ap.add_argument("--block-steps", type=int, default=0)
    ap.add_argument("--prefetch", type=int, default=0)
    ap.add_argument("--state-in-hbm", type=int, default=0)
    ap.add_argument("--rows", type=int, default=0)
    ap.add_argument("--helpers", type=int, default=0)
    ap.add_argument("--slices", type=int, default=0)
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of the benchmark, copy MIB MiB device to device three times and exit: "
                         "under `rocprofv3 --pmc FETCH_SIZE` (or WRITE_SIZE) each dispatch reads and writes "
                         "exactly that many bytes, which gives the counter's unit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; --gpus must be 1 "
              "(chains shard across GPUs with one all-reduce, which is not part of it)",
              file=sys.stderr)
        return 2

    import torch
    from paper_1708_04801_amd import api
    from paper_1708_04801_amd import workloads as wl

    api.load()          # raises if the HIP library is missing: there is no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    if args.calibrate_copy > 0:
        n = args.calibrate_copy * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration_copy_bytes_per_dispatch": n * 4, "dispatches": 3}))
        return 0

    if args.workload == "delay_servers":
        return bench_delay_servers(args, torch, api, wl)

    t_gen = time.time()
    w = wl.FULL[args.workload]()
    t_gen = time.time() - t_gen
    X = api.matrix_from_workload(w)
    y = torch.from_numpy(w.y).cuda()
    k, d = w.k, w.d
    plan = None
    if args.threads or args.block_steps or args.prefetch or args.state_in_hbm or args.rows or args.helpers or args.slices:
        plan = {"threads": args.threads, "block_steps": args.block_steps, "prefetch": args.prefetch,
                "state_in_hbm": args.state_in_hbm, "rows": args.rows, "helpers": args.helpers,
                "slices": args.slices}
    desc = api.wpsgd_describe_plan(X, k, w.loss, plan)
    W = torch.empty((k, d), dtype=torch.float32, device="cuda")
    v = torch.empty(d, dtype=torch.float32, device="cuda")
    ws_chain = torch.empty(max(256, api.wpsgd_run_chains_workspace(X, k, w.loss, plan)), dtype=torch.uint8,
                           device="cuda")
    ws_comb = torch.empty(max(256, api.wpsgd_combine_workspace(k, d)), dtype=torch.uint8, device="cuda")

    def step(ev=None):
        if ev is not None:
            ev[0].record()
        api.wpsgd_run_chains(X, y, w.n_steps, w.eta, w.lam, w.loss, w.seed, W=W, workspace=ws_chain, plan=plan)
        if ev is not None:
            ev[1].record()
        a = api.wpsgd_weights(w.n_steps, w.eta, w.lam)
        api.wpsgd_combine(W, a, w_out=v, workspace=ws_comb)
        if ev is not None:
            ev[2].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    total_updates = int(w.n_steps.sum())
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    chain_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    combine_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    # algorithmic bytes of one sample-update: the stored row plus its 4-byte label; CSR adds the
    # two row offsets and the gather + scatter of the touched model entries (4 bytes each way)
    if w.is_csr:
        nnz = w.vals.size / w.m
        bytes_per_update = nnz * 8 + 16 + 4 + nnz * 8
    else:
        bytes_per_update = w.row_bytes() + 4
    algo_bytes = bytes_per_update * total_updates
    achieved = algo_bytes / (chain_ms * 1e-3) / 1e9
    traffic = measured_traffic(args.workload) if plan is None else None

    out = {
        "metric": "SGD sample-updates/sec (all chains)",
        "value": total_updates / (ms_per_step * 1e-3),
        "unit": "sample-updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.loss == wl.LOGISTIC else "f64",
        "data": "synthetic",
        "config": {"workload": args.workload, "m": w.m, "d": d, "k": k, "sample_updates_per_step": total_updates,
                   "storage": "csr" if w.is_csr else ("bf16" if w.is_bf16 else "f32"),
                   "loss": "hinge" if w.loss == wl.HINGE else "logistic", "kernel": desc,
                   "imbalance_mean_over_max": float(w.n_steps.mean() / max(1, w.n_steps.max()))},
        "roofline": {"bound": "hbm", "kernel": "chain kernel (wpsgd_run_chains)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "bytes_per_sample_update": bytes_per_update,
                     "kernel_ms": chain_ms, "combine_ms": combine_ms,
                     # a chain is sequential: the launch lasts as long as its longest chain, so this
                     # per-step time is what sets the achieved bandwidth
                     "longest_chain_steps": int(w.n_steps.max()),
                     "us_per_step_longest_chain": chain_ms * 1e3 / max(1, int(w.n_steps.max()))},
        "data_generation_s": t_gen,
    }

    # What the shape of the workload allows.  A chain is a sequential recursion and all chains step at
    # about one rate.  When every chain has a compute unit from the start (k <= 256), the launch lasts as
    # long as its longest chain and chain i is alive for n_i / max n of it: averaged over the launch the
    # kernel cannot draw more than mean(n)/max(n) of what the whole chip streams.  With more chains than
    # compute units, finished chains are replaced by waiting ones and the factor does not apply.  The
    # streaming figure is measured here (many workgroups reading rows in sample order, no arithmetic): a
    # yardstick, not a law; a kernel whose access pattern suits the memory system better can pass it.
    imbalance = float(w.n_steps.mean() / max(1, w.n_steps.max()))
    all_resident = k <= 256
    shape = {"alive_fraction": imbalance if all_resident else 1.0, "all_chains_resident_from_the_start": all_resident}
    # probes: rows of the workload's own size when they are 16 KiB or longer, and the same buffer (CSR: the
    # values array) seen as rows of 16 KiB; the better of the two counts
    views = []
    if not w.is_csr and w.row_bytes() >= 16384 and w.row_bytes() % 16 == 0:
        views.append(X.dense)
    flat = (X.vals if w.is_csr else X.dense).reshape(-1)
    per_row = 16384 // flat.element_size()
    flat = flat[: flat.numel() // per_row * per_row].view(-1, per_row)
    if flat.dtype not in (torch.float32, torch.bfloat16):
        flat = flat.view(torch.float32)
    views.append(flat)
    stream_gbs, streamed_row_bytes = None, None
    for view in views:
        if view.shape[0] < 1024:
            continue
        Xs = api.Matrix(view.shape[0], view.shape[1], dense=view)
        row_b = view.shape[1] * view.element_size()
        groups = 1024
        rows = int(max(16, (1 << 31) // (groups * row_b)))
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            api.wpsgd_stream_rows(Xs, groups, rows)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        gbs = groups * rows * row_b / (best * 1e-3) / 1e9
        if stream_gbs is None or gbs > stream_gbs:
            stream_gbs, streamed_row_bytes = gbs, row_b
    if stream_gbs is not None:
        shape.update({"whole_chip_streaming_GBps": stream_gbs, "streamed_row_bytes": streamed_row_bytes,
                      "attainable_GBps": stream_gbs * shape["alive_fraction"],
                      "frac_of_attainable": achieved / (stream_gbs * shape["alive_fraction"])})
    out["roofline"]["shape_bound"] = shape

    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        Xo = orc.CSR(w.row_ptr, w.col_idx, w.vals, w.d) if w.is_csr else orc.Dense(w.dense)
        cores = min(k, len(os.sched_getaffinity(0)))
        n_cpu, sample = w.n_steps, "the whole workload, all chains in full"
        csr_mode, mode_name = orc.PLAIN, "plain"
        if args.workload == "sparse_hinge":
            csr_mode, mode_name = orc.LAZY, "scalar-scale (the literal shrink touches 2^20 doubles a step)"
        tc = time.perf_counter()
        Wo, _ = orc.run_chains(Xo, w.y, n_cpu, w.eta, w.lam, w.loss, w.seed, csr_mode=csr_mode, threads=cores)
        a = orc.weights(n_cpu, w.eta, w.lam)
        vo = orc.combine(Wo, a)
        tc = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": float(n_cpu.sum()) / tc, "unit": "sample-updates/s", "cores": cores,
                               "kind": "oracle", "sample": sample, "mode": mode_name, "seconds": tc}
        vg = v.cpu().numpy().astype(np.float64)
        out["parity_rel_l2"] = float(np.linalg.norm(vg - vo) / max(np.linalg.norm(vo), 1e-300))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
