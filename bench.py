#!/usr/bin/env python3
"""Benchmark of the hot path: ensemble multiplicative-update iterations of non-negative RESCAL.

One "step" = one ensemble iteration (Alg. 3's outer loop body for all q members at one rank k, with the
perturbation of Alg. 4 fused into the pass over X), on synthetic data shaped like the paper's workloads.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c1|c2|c3|c4|c4s|c5] [--k RANK] [--no-cpu]

The default workload is the dense medium configuration (n=2048, m=16, q=20, delta=0.03) at k=16.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by what the
# same counters read for a plain 1 GiB copy (profiles/dense_stream_c2_k16.txt, profiles/spmm_gather_c4_k32.txt,
# profiles/update_kernels_c5_k64.txt);
# keyed by (workload, k)
MEASURED_TRAFFIC_BYTES = {("c2", 16): 874.0e6, ("c3", 16): 113.2e9, ("c4", 32): 5079.0e6, ("c5", 64): 9032.0e6}


def make_workload(name, k_arg, device=None):
    """Returns (description dict, input, kind); kind in {"dense", "dense_device", "sparse", "sparse_csr"}.  The dense large
    tensor (34 GB) is built on the device; everything else on the host."""
    from synth import generators as gen
    if name == "c1":
        X, _, _ = gen.dense_tiny()
        return dict(workload="dense tiny n=64 m=4 planted rank 3", n=64, m=4, q=5, k=k_arg or 3, delta=0.03), X, "dense"
    if name == "c2":
        X, _, _ = gen.dense_community(n=2048, m=16, rank=8, noise=0.01, seed=0)
        return dict(workload="dense medium n=2048 m=16 planted rank 8, 1% noise", n=2048, m=16, q=20, k=k_arg or 16,
                    delta=0.03), X, "dense"
    if name == "c3":
        from synth.device_generators import dense_community_device
        X, _, _ = dense_community_device(16384, 32, 16, 0.01, 0, device)
        return dict(workload="dense large n=16384 m=32 planted rank 16, 1% noise (34 GB, built on the device)", n=16384,
                    m=32, q=8, k=k_arg or 16, delta=0.03), X, "dense_device"
    if name == "c5":
        S, _, _ = gen.sparse_powerlaw(n=10_000_000, m=4, draws_per_slice=50_000_000, rank=64, seed=0)
        return dict(workload="sparse power-law n=1e7 m=4, Zipf(1.1) rows and columns", n=S.n, m=S.m, q=2, k=k_arg or 64,
                    delta=0.03, nnz=S.nnz), S, "sparse"
    if name == "c4":
        S, _, _ = gen.sparse_community(n=1_000_000, m=8, nnz_per_slice=10_000_000, rank=32, communities=32, seed=0)
        return dict(workload="sparse n=1e6 m=8 ~1e7 nnz/slice, 32 communities, given as CSR (the library builds its "
                             "CSC copy at init)", n=S.n, m=S.m, q=4, k=k_arg or 32, delta=0.03, nnz=S.nnz), S, "sparse_csr"
    if name == "c4s":   # the same tensor with the entity ids shuffled: no locality in the gathers
        S, _, _ = gen.sparse_community(n=1_000_000, m=8, nnz_per_slice=10_000_000, rank=32, communities=32, seed=0,
                                       shuffle_ids=True)
        return dict(workload="sparse n=1e6 m=8 ~1e7 nnz/slice, 32 communities, entity ids shuffled", n=S.n, m=S.m, q=4,
                    k=k_arg or 32, delta=0.03, nnz=S.nnz), S, "sparse"
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(desc, X_host, kind, budget_s=20.0):
    """The CPU oracle as it stands, on a bounded sample: ONE ensemble member, all slices, a few iterations.
    Scaled to the metric's unit (ensemble iterations/s = member iterations/s divided by q)."""
    import numpy as np
    from oracle import mu, perturb
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    n, m, k, q = desc["n"], desc["m"], desc["k"], desc["q"]
    scale, note = 1.0, f"all {m} slices"
    if kind == "dense_device":
        # the tensor lives on the GPU: time the oracle on the leading nb x nb block of slice 0 and scale by the
        # n^2 m cost of an iteration
        nb = 4096
        X_host = X_host[0, :nb, :nb].cpu().numpy()[None]
        scale, note = (nb / n) ** 2 / m, f"leading {nb}x{nb} block of 1 of {m} slices, time scaled by (n/{nb})^2*m"
        n, m, kind = nb, 1, "dense"
    if kind == "dense":
        Xq = list(perturb.perturb_dense(X_host, 0, 0, desc["delta"]))
    else:
        from oracle import select
        Xq = select.perturbed_members(X_host.to_scipy(), 0, 1, desc["delta"])[0]
    A = perturb.init_A(0, 0, n, k)
    R = perturb.init_R(0, 0, m, k)
    A, R = mu.mu_iteration(Xq, A, R)            # untimed first call
    iters, t0 = 0, time.perf_counter()
    while True:
        A, R = mu.mu_iteration(Xq, A, R)
        iters += 1
        el = time.perf_counter() - t0
        if el > budget_s or iters >= 200:
            break
    member_it_s = iters / el * scale
    return {"value": member_it_s / q, "unit": "ensemble MU iterations/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 of {q} members, {note}, {iters} fp64 iterations in {el:.1f} s "
                      f"({member_it_s:.4g} member-iterations/s, divided by q)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--k", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--delta", type=float, default=None, help="perturbation half-width (default: the workload's, 0.03)")
    ap.add_argument("--q", type=int, default=0, help="ensemble size (default: the workload's)")
    ap.add_argument("--check-every", type=int, default=0,
                    help="time nnrescal_fit_until with a threshold that is never met, checking the error of Eq. 1 "
                         "every N iterations (0: plain nnrescal_fit, the default)")
    ap.add_argument("--start-rounds", type=int, default=0,
                    help="start from the SVD-based start with this many subspace rounds instead of the random start; "
                         "its wall time is reported as config.start_ms (it lies outside the timed steps)")
    ap.add_argument("--no-profile", action="store_true",
                    help="no per-launch events in the timed region (tensors small enough then take the single-launch "
                         "kernel); the roofline figures then come from the ten extra iterations after it")
    ap.add_argument("--copy-calib", action="store_true",
                    help="only run a plain device copy of 1 GiB (to calibrate the HBM traffic counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2202_09512_amd as nn
    nn.load()                                    # fails loudly if the HIP library is missing
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    dev = torch.device("cuda:0")
    if args.copy_calib:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read, 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 4 << 28, "copy_bytes_written": 4 << 28, "copies": 3}))
        return
    desc, X_host, kind = make_workload(args.workload, args.k, dev)
    torch.cuda.synchronize()                     # inputs are complete before another stream reads them
    if args.delta is not None:
        desc["delta"] = args.delta
    if args.q:
        desc["q"] = args.q
    n, m, k, q = desc["n"], desc["m"], desc["k"], desc["q"]
    if kind == "dense":
        X = nn.DenseX(torch.from_numpy(X_host).to(dev))
    elif kind == "dense_device":
        X = nn.DenseX(X_host)
    else:
        X = nn.SparseX.from_host(X_host, dev, with_csc=(kind != "sparse_csr"))
    stream = torch.cuda.Stream(device=dev)
    h = nn.nnrescal_init(X, k=k, q=q, delta=desc["delta"], eps_div=1e-16, seed=0, stream=stream)
    start_ms = None
    if args.start_rounds > 0:
        torch.cuda.synchronize()
        t_s = time.perf_counter()
        nn.nnrescal_start_nndsvd(h, args.start_rounds, 10, 0.01)
        torch.cuda.synchronize()
        start_ms = (time.perf_counter() - t_s) * 1e3
    nn.nnrescal_fit(h, args.warmup)
    stream.synchronize()
    torch.cuda.synchronize()

    # timed region: exactly `steps` ensemble iterations, events on the stream the kernels run on; inside it only
    # the dominant kernels (the passes over X) are bracketed by events of their own
    nn.nnrescal_profile(h, 0 if args.no_profile else 2)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    if args.check_every > 0:
        nn.nnrescal_fit_until(h, args.steps, 0.0, args.check_every)
    else:
        nn.nnrescal_fit(h, args.steps)
    ev1.record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = nn.nnrescal_profile(h, True)
    # the break-down over all kernel classes comes from a few more iterations outside the timed region
    class_steps = min(args.steps, 10)
    nn.nnrescal_fit(h, class_steps)
    prof_all = nn.nnrescal_profile(h, False)
    if args.no_profile:
        prof = prof_all
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    # with per-launch events on, the wall clock is the honest (slightly pessimistic) figure
    ms_per_step = max(ms_per_step, wall * 1e3 / args.steps)
    obj, xn = nn.nnrescal_objective(h)
    nn.nnrescal_destroy(h)

    it_s = 1e3 / ms_per_step
    if not kind.startswith("sparse"):
        bytes_alg = 4.0 * m * n * n                       # X read once for all members
        qbig = 8 if k <= 16 else (4 if k <= 32 else 2)   # members per group of the dense pass
        full_members = (q // qbig) * qbig
        ms_k, launches = prof["matrix_mul"]
        if launches == 0:                                 # q < 8: only the tail-group kernel runs
            ms_k, launches = prof["matrix_mul_tail"]
            full_members = q
        flops_launch = 4.0 * m * n * n * k * full_members  # two n^2 k contractions per member, 2 flops per FMA
        avg_ms = ms_k / max(launches, 1)
        roof = {"bound": "mfma", "kernel": f"dense_stream_kernel (groups of {qbig} members)",
                "achieved": flops_launch / (avg_ms * 1e-3) / 1e12, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "avg_launch_ms": avg_ms, "launches": int(launches), "members_per_launch": full_members,
                "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, k))}
    else:
        nnz = desc["nnz"]
        # rows of X_t A (X_t^T A) that exist at all: the entity rows (columns) of slice t with a non-zero; the
        # others are zero throughout and no algorithm has to move them
        rows_p = float(np.mean([(np.diff(X_host.csr_rowptr[t]) > 0).sum() for t in range(m)]))
        rows_q = float(np.mean([(np.diff(X_host.csc_colptr[t]) > 0).sum() for t in range(m)]))
        # per iteration: both formats of X once; per slice X_t A written once and read twice (A^T X_t A, A rule),
        # X_t^T A written once and read once; A read and written once
        bytes_alg = 16.0 * nnz + 4.0 * k * q * (m * (3 * rows_p + 2 * rows_q) + 2 * n)
        ms_k, launches = prof["matrix_mul_sparse"]
        # per launch (one product of one slice): one format of the slice once (index + value), the rows of A that
        # the slice refers to read once, the product's non-zero rows written once (the same sum for both products)
        per_launch = 8.0 * nnz / m + 4.0 * k * q * (rows_p + rows_q)
        avg_ms = ms_k / max(launches, 1)
        roof = {"bound": "hbm", "kernel": "spmm_gather_kernel (one product of one slice)",
                "achieved": per_launch / (avg_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "avg_launch_ms": avg_ms, "launches": int(launches),
                "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, k))}
    roof["frac"] = roof["achieved"] / roof["peak"]
    out = {
        "metric": "MU iterations/sec and achieved HBM TB/s (fraction of peak) per (n,m,k,q)",
        "value": it_s, "unit": "ensemble MU iterations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": dict(desc, eps_div=1e-16, member_iterations_per_s=it_s * q,
                       **({"check_every": args.check_every} if args.check_every > 0 else {}),
                       **({"timed_without_events": True} if args.no_profile else {}),
                       **({"start_rounds": args.start_rounds, "start_ms": start_ms} if start_ms is not None else {})),
        "hbm_alg_TBps": bytes_alg / (ms_per_step * 1e-3) / 1e12,
        "hbm_alg_frac": bytes_alg / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "kernel_class_ms_per_step": {c: v[0] / class_steps for c, v in prof_all.items()},
        "rel_error_member0": (max(obj[0], 0.0) / xn[0]) ** 0.5,
        "roofline": roof,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(desc, X_host, kind)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
