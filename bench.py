#!/usr/bin/env python3
"""Benchmark of the hot path: ensemble multiplicative-update iterations of non-negative RESCAL.

One "step" = one ensemble iteration (Alg. 3's outer loop body for all q members at one rank k, with the
perturbation of Alg. 4 fused into the pass over X), on synthetic data shaped like the paper's workloads.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|c1|c2|c3|c4|c4s|c5|bin] [--k RANK] [--no-cpu]

The headline line is the largest single-GPU configuration, dense large (n=16384, m=32, q=8, 34 GB) at k=16.  With the
default `--workload all` the other configurations (dense medium, sparse, sparse power-law, binary sparse) are timed
in the same run and reported under "configs", each with its own roofline and CPU-oracle figures.

Timing protocol: W warm-up steps, then exactly K steps, enqueued as `--repeats` equal groups that are bracketed by
events on the stream the kernels run on; ms_per_step is the time of all K steps divided by K, ms_per_step_median
the median over the groups.  The dominant kernels carry events of their own inside the timed region (the roofline
figures); the break-down over all kernel classes comes from ten more steps after it.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix
CSRC = os.path.join(ROOT, "paper_2202_09512_amd", "csrc")

# HBM bytes per launch of a kernel from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE), each scaled by what the same
# counter reads for a plain copy of known size (the summaries under profiles/ give the commands).  An entry is only
# reported while the kernel's source is the one that was measured (first 12 hex digits of its SHA-256): after a change
# to the kernel the figure reads null until the counters have been taken again.
RECORDED_TRAFFIC = {
    # (workload, k, kernel class): (bytes per launch, source file, sha256[:12] of that file, profile)
    ("c3", 16, "matrix_mul"): (102.39e9, "kernels_dense.hip", "3e10b5077a52", "profiles/dense_stream_c3_k16.txt"),
    ("c2", 16, "matrix_mul"): (0.869e9, "kernels_dense.hip", "3e10b5077a52", "profiles/dense_stream_c2_k16.txt"),
    ("c4", 32, "matrix_mul_sparse"): (44.78e9, "kernels_sparse.hip", "4f614c1e6a17", "profiles/spmm_gather_c4_k32.txt"),
    ("c5", 64, "matrix_mul_sparse"): (146.56e9, "kernels_sparse.hip", "4f614c1e6a17", "profiles/sparse_iteration_c5_k64.txt"),
}


def _sha12(path):
    with open(path, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:12]


def recorded_traffic(workload, k, cls, form=None):
    rec = RECORDED_TRAFFIC.get((workload, k, cls))
    if rec is None:
        return None, None
    if cls == "matrix_mul_sparse" and form != "lines":
        return None, f"{rec[3]} holds counters of the lines form of the products, this run used '{form}'"
    nbytes, src, sha, profile = rec
    if _sha12(os.path.join(CSRC, src)) != sha:
        return None, f"{profile} holds counters of an earlier version of {src}"
    return nbytes, profile


# ------------------------------------------------------------------------------------------------- workloads
def make_workload(name, k_arg, device):
    """Returns (description, host tensor or None, library tensor, kind); kind in {"dense", "sparse"}.  Large tensors
    are drawn on the device (synth/device_generators.py) and copied to the host for the oracle leg."""
    import torch
    import paper_2202_09512_amd as nn
    from synth import generators as gen
    from synth import device_generators as dgen
    if name == "c1":
        X, _, _ = gen.dense_tiny()
        return (dict(workload="dense tiny n=64 m=4 planted rank 3", n=64, m=4, q=5, k=k_arg or 3, delta=0.03), X,
                nn.DenseX(torch.from_numpy(X).to(device)), "dense")
    if name == "c2":
        X, _, _ = gen.dense_community(n=2048, m=16, rank=8, noise=0.01, seed=0)
        return (dict(workload="dense medium n=2048 m=16 planted rank 8, 1% noise", n=2048, m=16, q=20, k=k_arg or 16,
                     delta=0.03), X, nn.DenseX(torch.from_numpy(X).to(device)), "dense")
    if name == "c3":
        X, _, _ = dgen.dense_community_device(16384, 32, 16, 0.01, 0, device)
        return (dict(workload="dense large n=16384 m=32 planted rank 16, 1% noise (34 GB, built on the device)", n=16384,
                     m=32, q=8, k=k_arg or 16, delta=0.03), None, nn.DenseX(X), "dense")
    if name in ("c4", "c4s"):
        D, _, _ = dgen.sparse_community_device(1_000_000, 8, 10_000_000, 32, 32, 0, device, shuffle_ids=(name == "c4s"))
        what = ("entity ids shuffled" if name == "c4s" else "given as CSR (the library builds its CSC copy at init)")
        return (dict(workload=f"sparse n=1e6 m=8 ~1e7 nnz/slice, 32 communities, {what}", n=D.n, m=D.m, q=4,
                     k=k_arg or 32, delta=0.03, nnz=D.nnz), D, nn.SparseX.from_device(D, with_csc=(name == "c4s")),
                "sparse")
    if name == "c5":
        D, _, _ = dgen.sparse_powerlaw_device(10_000_000, 4, 127_000_000, 64, 0, device)
        return (dict(workload="sparse power-law n=1e7 m=4, Zipf(1.1) rows and columns, 1.27e8 draws per slice, CSR+CSC",
                     n=D.n, m=D.m, q=2, k=k_arg or 64, delta=0.03, nnz=D.nnz), D, nn.SparseX.from_device(D), "sparse")
    if name == "bin":
        D, _, _ = dgen.sparse_binary_device(1_000_000, 8, 10_000_000, 32, 0, device)
        return (dict(workload="binary sparse n=1e6 m=8 ~1e7 ones/slice, 32 communities, CSR without a value array",
                     n=D.n, m=D.m, q=4, k=k_arg or 32, delta=0.03, nnz=D.nnz), D,
                nn.SparseX.from_device(D, with_csc=False), "sparse")
    raise SystemExit(f"unknown workload {name}")


# ------------------------------------------------------------------------------------------------- CPU oracle
def cpu_baseline(desc, X_host, X_lib, kind, budget_s=8.0):
    """The CPU oracle as it stands on a bounded sample: ONE ensemble member and, for the large tensors, ONE slice
    (the slice loop is what an iteration consists of: its time is scaled by m), timed twice: with the BLAS thread pool
    at one thread, and with all host cores.  Scaled to the metric's unit (ensemble iterations/s = member iterations/s
    divided by q).  The member's perturbed tensor is built beforehand, as the method itself keeps it fixed."""
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import fast, mu
    n, m, k, q, delta = desc["n"], desc["m"], desc["k"], desc["q"], desc["delta"]
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    if kind == "dense":
        if X_host is None:          # the tensor lives on the GPU: slice 0 comes back to the host
            Xq = [fast.perturb_dense_slice(X_lib.X[0].cpu().numpy(), 0, 0, 0, delta)]
        elif m * n * n > (1 << 28):
            Xq = [fast.perturb_dense_slice(X_host[0], 0, 0, 0, delta)]
        else:
            Xq = [fast.perturb_dense_slice(X_host[t], t, 0, 0, delta) for t in range(m)]
    else:
        import scipy.sparse as sp
        S = X_host.to_host() if hasattr(X_host, "to_host") else X_host
        Xq = []
        for t in range(m if S.nnz <= 2_000_000 else 1):
            lo, hi = int(S.csr_slice_off[t]), int(S.csr_slice_off[t + 1])
            rows, cols, vals = S.slice_coo(t)
            Xq.append(sp.csr_matrix((fast.perturb_coo(rows, cols, vals, t, n, 0, 0, delta), S.csr_col[lo:hi],
                                     S.csr_rowptr[t]), shape=(n, n)))
    ms = len(Xq)
    scale = ms / m                                   # one of m slices timed: an iteration takes m times as long
    note = f"all {m} slices" if ms == m else f"{ms} of {m} slices, time scaled by {m // ms}"
    A0, R0 = fast.init_A(0, 0, n, k), fast.init_R(0, 0, ms, k)

    def timed(threads):
        with threadpool_limits(limits=threads):
            A, R = mu.mu_iteration(Xq, A0, R0)      # untimed first call
            iters, t0 = 0, time.perf_counter()
            while True:
                A, R = mu.mu_iteration(Xq, A, R)
                iters += 1
                el = time.perf_counter() - t0
                if el > budget_s or iters >= 200:
                    return iters / el * scale, iters, el
    all_rate, it_a, el_a = timed(cores)
    one_rate, it_1, el_1 = timed(1)
    return {"value": all_rate / q, "unit": "ensemble MU iterations/s", "cores": int(cores), "kind": "oracle",
            "single_thread_value": one_rate / q,
            "sample": f"1 of {q} members, {note}: {it_a} fp64 iterations in {el_a:.1f} s with {cores} threads "
                      f"({all_rate:.4g} member-iterations/s), {it_1} in {el_1:.1f} s with one thread "
                      f"({one_rate:.4g}); divided by q"}


# ------------------------------------------------------------------------------------------------- one configuration
def rows_with_entries(ptr_dev, m):
    """Per slice, the number of entity rows (columns) that hold a stored non-zero."""
    d = ptr_dev[:, 1:] - ptr_dev[:, :-1]
    return float((d > 0).sum().item()) / m


def run_config(name, args, steps, with_cpu):
    import torch
    import paper_2202_09512_amd as nn
    dev = torch.device("cuda:0")
    desc, X_host, X, kind = make_workload(name, args.k, dev)
    torch.cuda.synchronize()                     # inputs are complete before another stream reads them
    if args.delta is not None:
        desc["delta"] = args.delta
    if args.q:
        desc["q"] = args.q
    n, m, k, q = desc["n"], desc["m"], desc["k"], desc["q"]
    stream = torch.cuda.Stream(device=dev)
    h = nn.nnrescal_init(X, k=k, q=q, delta=desc["delta"], eps_div=1e-16, seed=0, stream=stream,
                         deterministic=args.deterministic, gather_form=args.gather_form)
    if kind != "dense":
        # which form of the sparse products runs (left to the library, it is chosen at init by timing them on the tensor)
        desc["gather_form"] = {0: "none", 1: "rows", 2: "lines"}[nn.nnrescal_gather_form(h)]
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

    # timed region: exactly `steps` ensemble iterations in `repeats` groups, events on the kernels' own stream
    repeats = max(1, min(args.repeats, steps))
    group = [steps // repeats + (1 if g < steps % repeats else 0) for g in range(repeats)]
    nn.nnrescal_profile(h, 0 if args.no_profile else 2)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(repeats + 1)]
    t0 = time.perf_counter()
    evs[0].record(stream)
    for g in range(repeats):
        if args.check_every > 0:
            nn.nnrescal_fit_until(h, group[g], 0.0, args.check_every)
        else:
            nn.nnrescal_fit(h, group[g])
        evs[g + 1].record(stream)
    stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = nn.nnrescal_profile(h, True)
    class_steps = min(steps, 10)
    nn.nnrescal_fit(h, class_steps)
    prof_all = nn.nnrescal_profile(h, False)
    if args.no_profile:
        prof = {c: (v[0] * steps / class_steps, v[1] * steps // class_steps) for c, v in prof_all.items()}
    per_group = [evs[g].elapsed_time(evs[g + 1]) / group[g] for g in range(repeats)]
    # with per-launch events on, the wall clock is the honest (slightly pessimistic) figure
    ms_per_step = max(evs[0].elapsed_time(evs[repeats]), wall * 1e3) / steps
    obj, xn = nn.nnrescal_objective(h)
    nn.nnrescal_destroy(h)

    class_ms = {c: v[0] / class_steps for c, v in prof_all.items()}
    if kind == "dense":
        bytes_alg = 4.0 * m * n * n                       # X read once for all members
        qbig = 8 if k <= 16 else (4 if k <= 32 else 2)   # members per group of the dense pass
        full_members = (q // qbig) * qbig
        ms_k, launches = prof["matrix_mul"]
        cls = "matrix_mul"
        if launches == 0:                                 # q < qbig: only the tail-group kernel runs
            ms_k, launches = prof["matrix_mul_tail"]
            full_members, cls = q, "matrix_mul_tail"
        flops_launch = 4.0 * m * n * n * k * full_members  # two n^2 k contractions per member, 2 flops per FMA
        avg_ms = ms_k / max(launches, 1)
        traffic, source = recorded_traffic(name, k, cls)
        roof = {"bound": "mfma", "kernel": f"dense_stream_kernel (groups of {qbig} members, all slices in one launch)",
                "achieved": flops_launch / (avg_ms * 1e-3) / 1e12, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "avg_launch_ms": avg_ms, "launches": int(launches), "members_per_launch": full_members,
                "traffic": traffic, "traffic_source": source}
    else:
        nnz = desc["nnz"]
        val_bytes = 0.0 if name == "bin" else 4.0         # a binary tensor has no value array
        # rows of X_t A (X_t^T A) that exist at all: the entity rows (columns) of slice t with a non-zero; the
        # others are zero throughout and no algorithm has to move them
        rows_p = rows_with_entries(X_host.csr_rowptr, m)
        rows_q = rows_with_entries(X_host.csc_colptr, m)
        # per iteration: both formats of X once; per slice X_t A written once and read twice (A^T X_t A, A rule),
        # X_t^T A written once and read once; A read and written once
        bytes_alg = 2 * (4.0 + val_bytes) * nnz + 4.0 * k * q * (m * (3 * rows_p + 2 * rows_q) + 2 * n)
        # algorithmic bytes per ITERATION of the three kernel classes that make up a sparse iteration; the class that
        # takes most of the iteration is the one the roofline is given for
        per_class_alg = {
            # the two products of every slice: both formats of X once, the rows of A that a slice refers to once per
            # slice and product, the products' rows that exist written once
            "matrix_mul_sparse": 2 * (4.0 + val_bytes) * nnz + 4.0 * k * q * m * 2 * (rows_p + rows_q),
            # the A rule: X_t A and X_t^T A of every slice (rows that exist) read once, A read and written once
            "a_rule": 4.0 * k * q * (m * (rows_p + rows_q) + 2 * n),
            # A^T X_t A for all slices: X_t A (rows that exist) once per slice, A once
            "gram_mul": 4.0 * k * q * (m * rows_p + n),
        }
        cls = max(per_class_alg, key=lambda c: class_ms.get(c, 0.0))
        timed = prof[cls] if prof[cls][1] else (prof_all[cls][0] * steps / class_steps, prof_all[cls][1] * steps // class_steps)
        launches_per_step = timed[1] / steps
        avg_ms = timed[0] / max(timed[1], 1)
        gather = "spmm_gather_lines_kernel" if desc.get("gather_form") == "lines" else "spmm_gather_kernel"
        kernel = {"matrix_mul_sparse": gather + " (X_t A and X_t^T A of all slices in one launch)",
                  "a_rule": "a_update16 kernels (Eq. 2's second rule over all slices)",
                  "gram_mul": "gram16_kernel (A^T X_t A of all slices)"}[cls]
        traffic, source = recorded_traffic(name, k, cls, desc.get("gather_form"))
        roof = {"bound": "hbm", "kernel": kernel,
                "achieved": per_class_alg[cls] / max(launches_per_step, 1e-9) / (avg_ms * 1e-3) / 1e9,
                "peak": PEAK_HBM_GBS, "unit": "GB/s", "avg_launch_ms": avg_ms, "launches": int(timed[1]),
                "launches_per_step": launches_per_step, "traffic": traffic, "traffic_source": source,
                "class_hbm_alg_frac": {c: per_class_alg[c] / (class_ms[c] * 1e-3) / 1e9 / PEAK_HBM_GBS
                                       for c in per_class_alg if class_ms.get(c, 0) > 0}}
    roof["frac"] = roof["achieved"] / roof["peak"]
    it_s = 1e3 / ms_per_step
    out = {
        "value": it_s, "unit": "ensemble MU iterations/s", "steps": steps, "warmup": args.warmup, "repeats": repeats,
        "ms_per_step": ms_per_step, "ms_per_step_median": float(np.median(per_group)),
        "ms_per_step_groups": [round(v, 4) for v in per_group],
        "dtype": "f32",
        "config": dict(desc, eps_div=1e-16, member_iterations_per_s=it_s * q,
                       **({"check_every": args.check_every} if args.check_every > 0 else {}),
                       **({"timed_without_events": True} if args.no_profile else {}),
                       **({"deterministic": True} if args.deterministic else {}),
                       **({"start_rounds": args.start_rounds, "start_ms": start_ms} if start_ms is not None else {})),
        "hbm_alg_TBps": bytes_alg / (ms_per_step * 1e-3) / 1e12,
        "hbm_alg_frac": bytes_alg / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "kernel_class_ms_per_step": class_ms,
        "rel_error_member0": (max(obj[0], 0.0) / xn[0]) ** 0.5,
        "roofline": roof,
    }
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(desc, X_host, X, kind)
    del X, X_host, h
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--repeats", type=int, default=5, help="the timed steps are enqueued as this many equal groups")
    ap.add_argument("--workload", default="all",
                    help="all (default: the headline configuration c3, then c2, c4, c5 and bin under 'configs') or one of "
                         "c1, c2, c3, c4, c4s, c5, bin")
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
    ap.add_argument("--deterministic", action="store_true",
                    help="time the reproducible mode (sums in a fixed order instead of atomic additions)")
    ap.add_argument("--gather-form", type=int, default=0,
                    help="sparse products: 0 = the library chooses (default), 1 whole rows, 2 one 128-byte line "
                         "of every factor row per pass")
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
    if args.copy_calib:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB read, 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 4 << 28, "copy_bytes_written": 4 << 28, "copies": 3}))
        return
    head_name = "c3" if args.workload == "all" else args.workload
    head = run_config(head_name, args, args.steps, not args.no_cpu)
    out = {
        "metric": "MU iterations/sec and achieved HBM TB/s (fraction of peak) per (n,m,k,q)",
        "value": head["value"], "unit": head["unit"], "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        # the paper prints no iterations/s for this path; the one figure that can be derived from its text, for context
        # only (another machine, another tensor): section "Model Determination in Large Data", a 20 x 396800 x 396800 dense
        # tensor, k = 2..11, 10 perturbations, 200 iterations in about 3 hours on 4096 CPU cores
        "paper_context": "about 1.9 member-iterations/s (derived: 20 000 member-iterations in ~3 h incl. clustering) on 4096 "
                         "Xeon cores for a dense 20 x 396800^2 tensor, k = 2..11; not comparable, not a target",
    }
    out.update({k: v for k, v in head.items() if k not in out})
    if args.workload == "all":
        # the other configurations, each timed the same way in this run (dense medium has short steps: five times as many)
        out["configs"] = {}
        for name, steps in (("c2", 5 * args.steps), ("c4", args.steps), ("c5", args.steps), ("bin", args.steps)):
            try:
                out["configs"][name] = run_config(name, args, steps, not args.no_cpu)
            except Exception as err:             # one configuration failing must not cost the headline line
                out["configs"][name] = {"error": f"{type(err).__name__}: {err}"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
