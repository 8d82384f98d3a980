#!/usr/bin/env python3
"""Benchmark of the MU NMF hot path on one MI355X.

Default workload (the one the headline metric is quoted on): dense fp32 A
32768 x 16384 (2 GiB, resident in HBM), planted rank 32 with multiplicative
U[0.95, 1.05) noise, k = 32, W and H ~ U[0, 1).  One step = one MU iteration
(H update then W update: W^T W, W^T A, H update, H H^T, A H^T with the fused W
update), i.e. two full reads of A.

Prints ONE JSON line on stdout.  Other workloads (--workload c1|c3|c3ooc|c4|c5|oom1|ck) are
there for the other measurements of this repository; they print the same kind
of line with their own unit.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
# HBM bytes per launch of the two streaming pass kernels on the default workload (row plan), from
# the FETCH_SIZE / WRITE_SIZE counters in profiles/dense_c2_hbm_traffic_pmc.txt (scaled by the
# plain-copy calibration stated there); only reported when that workload is the one timed.
C2_PASS_TRAFFIC_BYTES = {"wta_pass": (1073365.2 * 2.0 + 8208.6) * 1024.0, "aht_pass": (1112235.3 * 2.0 + 4437.3) * 1024.0}
# HBM bytes per iteration of the sparse workload c3 (both gather launches), from the counters in
# profiles/csr_c3_hbm_traffic_pmc.txt (scaled by the plain-copy calibration stated there).
C3_ITERATION_TRAFFIC_BYTES = (30746040.6 + 30666910.4) * 2.0 * 1024.0 + (131072.0 + 524328.3) * 1024.0
EPS = 1e-16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def sync_time(torch):
    torch.cuda.synchronize()
    return time.perf_counter()


def cpu_baseline_dense(A_host, k, seed, iters=3):
    """The oracle as it stands, on the host cores, on the full matrix for a
    few iterations (its cost per iteration does not depend on the iterate)."""
    import nmf_inputs
    from oracle import nmf_oracle as orc
    m, n = A_host.shape
    W, H = nmf_inputs.init_factors(m, n, k, seed)
    W, H = W.numpy(), H.numpy()
    t0 = time.perf_counter()
    orc.mu_dense(A_host, W, H, iters, EPS)
    dt = time.perf_counter() - t0
    return {"value": iters / dt, "unit": "iterations/s", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{iters} iterations of the full {m}x{n}, k={k} workload in {dt:.1f} s (float64)"}


def flops_per_iteration(m, n, k):
    """Operation count of one iteration in the paper's model (section 3.1, its rows I = m):
    W^T A, W^T W, the element-wise H update, H H^T, W (H H^T), A H^T, the element-wise W update,
    with the first addition of every sum counted as free, plus the (W^T W) H product (2 k k n)
    that the model's list leaves out."""
    listed = 2 * k * m * n + 2 * k * m * k + 2 * k * n + 2 * k * n * k + 2 * m * k * k + 2 * m * n * k + 2 * m * k \
        - k * n - 2 * k * k - 2 * m * k
    return listed + 2 * k * k * n


def bench_c2(args, torch, nmf, nmf_inputs, m=32768, n=16384, k=32, rank=32, tag="c2"):
    A = nmf_inputs.dense_planted(m, n, rank, seed=1002, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2002, device="cuda")
    log(f"[bench] {tag}: A {m}x{n} fp32 ({A.numel() * 4 / 2**30:.2f} GiB), k={k}")
    if args.calibrate:
        # a plain device copy of known size (reads and writes A.numel()*4 bytes), for scaling
        # the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run
        B = torch.empty_like(A)
        B.copy_(A)
        torch.cuda.synchronize()
        del B
    if args.warmup:
        nmf.nmf_mu_dense(A, m, n, k, W, H, args.warmup, EPS)
    t0 = sync_time(torch)
    nmf.nmf_mu_dense(A, m, n, k, W, H, args.steps, EPS)
    t1 = sync_time(torch)
    ms_step = (t1 - t0) * 1e3 / args.steps
    assert bool(torch.isfinite(W).all()) and bool(torch.isfinite(H).all())
    # per-kernel times with HIP events between the launches, same launch configuration
    names = ["gram_w", "wta_pass", "h_update", "gram_h", "aht_pass", "w_update"]
    kms = nmf.nmf_mu_dense_profile(A, m, n, k, W, H, min(args.steps, 50), EPS)
    kern = dict(zip(names, kms[:6]))
    plan = {0: "small (direct A H^T kernel)", 1: "mirrored (A and A^T resident)", 2: "row plan (both passes stream the row-major A)"}[int(kms[6])]
    log("[bench] plan:", plan)
    log("[bench] per-kernel ms:", {a: round(b, 4) for a, b in kern.items()})
    # the two pass kernels alone: 20 launches back to back between two HIP events on their
    # stream (the per-kernel figures above carry the event commands around every launch)
    alone = {"wta_pass": kms[7], "aht_pass": kms[8]}
    log("[bench] pass kernels, back-to-back launches, ms:", {a: round(b, 4) for a, b in alone.items()})
    timed = {a: (alone[a] if alone[a] > 0 else kern[a]) for a in alone}
    dom = max(timed, key=lambda x: timed[x])
    bytes_a = m * n * 4          # one pass reads every element of A once: 4 B per element
    ach = bytes_a / (timed[dom] * 1e-3) / 1e9
    gbs_iter = 2 * bytes_a / (ms_step * 1e-3) / 1e9
    out = {
        "metric": "MU iterations/s (dense fp32, resident A)", "value": 1e3 / ms_step, "unit": "iterations/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{tag}: dense fp32 A {m}x{n} resident, planted rank {rank} x U[0.95,1.05), k={k}, "
                               "one step = one MU iteration (2 reads of A)", "m": m, "n": n, "k": k, "plan": plan},
        "gbs_over_A": gbs_iter, "frac_hbm_peak_over_A": gbs_iter / HBM_PEAK_GBS,
        "tflops_paper_model": flops_per_iteration(m, n, k) / (ms_step * 1e-3) / 1e12,
        "kernel_ms": kern, "pass_kernel_ms_back_to_back": alone,
        "roofline": {"bound": "hbm", "kernel": dom, "kernel_ms": timed[dom], "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": ach / HBM_PEAK_GBS,
                     "traffic": C2_PASS_TRAFFIC_BYTES[dom] if (m, n, k, int(kms[6])) == (32768, 16384, 32, 2) else None,
                     "algorithmic_bytes_per_launch": bytes_a},
    }
    # the objective ||A - W H||_F in row tiles (one more streaming pass over A), blocking call
    nmf.nmf_residual_dense(A, m, n, k, W, H)
    t0 = time.perf_counter()
    for _ in range(5):
        res = nmf.nmf_residual_dense(A, m, n, k, W, H)
    dt = (time.perf_counter() - t0) / 5
    out["objective"] = {"residual_fro": res, "ms": dt * 1e3, "gbs_over_A": bytes_a / dt / 1e9}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_dense(A.cpu().numpy(), k, seed=2002)
    return out


def bench_c1(args, torch, nmf, nmf_inputs):
    m, n, k = 256, 192, 4
    A = nmf_inputs.dense_planted(m, n, 4, seed=1001, noise="add", lo=0.0, hi=0.01).cuda()
    W, H = (t.cuda() for t in nmf_inputs.init_factors(m, n, k, seed=2001))
    nmf.nmf_mu_dense(A, m, n, k, W, H, max(args.warmup, 1), EPS)
    t0 = sync_time(torch)
    nmf.nmf_mu_dense(A, m, n, k, W, H, args.steps, EPS)
    t1 = sync_time(torch)
    ms_step = (t1 - t0) * 1e3 / args.steps
    out = {"metric": "MU iterations/s (dense fp32, launch bound)", "value": 1e3 / ms_step, "unit": "iterations/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "c1: dense 256x192, k=4"},
           # the whole problem (192 KiB) lives in cache: the iteration is a chain of dependent launches
           "roofline": {"bound": "launch latency", "achieved": None, "peak": None, "unit": None, "frac": None,
                        "traffic": None, "launches_per_iteration": 4}}
    if not args.no_cpu_baseline:
        from oracle import nmf_oracle as orc
        Ah = A.cpu().numpy()
        W0, H0 = (t.numpy() for t in nmf_inputs.init_factors(m, n, k, seed=2001))
        t0 = time.perf_counter()
        orc.mu_dense(Ah, W0, H0, 100, EPS)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 100 / dt, "unit": "iterations/s", "cores": orc.num_threads(), "kind": "oracle",
                               "sample": f"all 100 iterations of the 256x192, k=4 workload in {dt * 1e3:.0f} ms (float64)"}
    return out


def bench_c3(args, torch, nmf, nmf_inputs):
    m, n, k, density = 4194304, 1048576, 32, 1e-4
    if args.small:
        m, n = m // 16, n // 16
        density *= 16
    t0 = time.perf_counter()
    rowptr, colidx, vals = nmf_inputs.csr_uniform(m, n, density, seed=1003, device="cuda")
    nnz = int(vals.numel())
    W, H = nmf_inputs.init_factors(m, n, k, seed=2003, device="cuda")
    log(f"[bench] c3: CSR {m}x{n}, nnz={nnz} ({nnz / m:.1f} per row), generated in {time.perf_counter() - t0:.1f} s")
    if args.calibrate:
        # a plain device copy of known size (reads and writes 4 nnz bytes), for scaling the
        # FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run
        B = torch.empty_like(vals)
        B.copy_(vals)
        torch.cuda.synchronize()
        del B
    nmf.nmf_mu_csr(rowptr, colidx, vals, m, n, nnz, k, W, H, max(args.warmup, 1), EPS)
    t0 = sync_time(torch)
    nmf.nmf_mu_csr(rowptr, colidx, vals, m, n, nnz, k, W, H, args.steps, EPS)
    t1 = sync_time(torch)
    ms_step = (t1 - t0) * 1e3 / args.steps
    # the same iterations with the objective of every iteration reported
    # (not part of the timed step): two calls of the same length, one plain, one monitored, so that
    # the set-up of a call, which both pay, drops out of the difference
    mon_iters = min(args.steps, 20)
    t2 = sync_time(torch)
    nmf.nmf_mu_csr(rowptr, colidx, vals, m, n, nnz, k, W, H, mon_iters, EPS)
    t3 = sync_time(torch)
    obj = nmf.nmf_mu_csr_monitor(rowptr, colidx, vals, m, n, nnz, k, W, H, mon_iters, EPS)
    t4 = sync_time(torch)
    mon_extra_ms = ((t4 - t3) - (t3 - t2)) * 1e3 / mon_iters
    log(f"[bench] c3 monitored: {mon_extra_ms:.2f} ms more per iteration than the plain run, objective {obj[-1]:.6g}")
    bytes_a = 2 * (8 * nnz + 8 * (m + 1))       # both passes read values, column indices, row pointers
    gbs = bytes_a / (ms_step * 1e-3) / 1e9
    gather = 2 * nnz * k * 4 + bytes_a
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle on the first 1/16 of the rows (same H, a sixteenth of A and W), a few iterations
        from oracle import nmf_oracle as orc
        ms_ = m // 16
        rp = rowptr[:ms_ + 1].cpu().numpy()
        e1 = int(rp[-1])
        ci, va = colidx[:e1].cpu().numpy(), vals[:e1].cpu().numpy()
        W0, H0 = (t.cpu().numpy() for t in nmf_inputs.init_factors(ms_, n, k, seed=2003, device="cuda"))
        t0 = time.perf_counter()
        orc.mu_csr(rp, ci, va, ms_, n, W0, H0, 2, EPS)
        dt = time.perf_counter() - t0
        cpu = {"value": 2 / dt / 16, "unit": "iterations/s", "cores": orc.num_threads(), "kind": "oracle",
               "sample": f"2 iterations on the first {ms_} rows ({e1} stored entries, 1/16 of the matrix) in {dt:.1f} s, "
                         "scaled by 1/16 to the whole matrix (float64)"}
    out_c3 = {"cpu_baseline": cpu} if cpu else {}
    return {**out_c3, "metric": "MU iterations/s (CSR fp32)", "value": 1e3 / ms_step, "unit": "iterations/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"c3: CSR {m}x{n}, nnz={nnz}, k={k}", "nnz": nnz},
            "gbs_over_A": gbs, "frac_hbm_peak_over_A": gbs / HBM_PEAK_GBS,
            # what the two gathers move: one k-float row of a factor per stored entry and product
            # (the tables, 128 MiB and 512 MiB here, do not fit the 4 MiB of L2 an XCD has)
            "roofline": {"bound": "hbm", "kernel": "aht_csr_kernel", "achieved": gather / (ms_step * 1e-3) / 1e9,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gather / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic": C3_ITERATION_TRAFFIC_BYTES if (m, n, k) == (4194304, 1048576, 32) else None,
                         "algorithmic_bytes_per_iteration": gather},
            "objective": {"residual_fro": obj[-1], "iterations": mon_iters,
                          "ms_more_per_monitored_iteration": mon_extra_ms}}


def bench_c3ooc(args, torch, nmf, nmf_inputs):
    """Config 3's matrix kept in pinned host memory and streamed in batches of 32 Mi stored entries."""
    m, n, k, density = 4194304, 1048576, 32, 1e-4
    if args.small:
        m, n = m // 16, n // 16
        density *= 16
    rowptr, colidx, vals = nmf_inputs.csr_uniform(m, n, density, seed=1003, device="cuda")
    nnz = int(vals.numel())
    rp, ci, va = rowptr.cpu().pin_memory(), colidx.cpu().pin_memory(), vals.cpu().pin_memory()
    del rowptr, colidx, vals
    W, H = nmf_inputs.init_factors(m, n, k, seed=2003, device="cuda")
    batch_nnz, budget = 32 << 20, 2 << 30
    # bare copy ceiling: the same three arrays in chunks of the batch size, one stream
    dci = torch.empty(batch_nnz, dtype=torch.int32, device="cuda")
    dva = torch.empty(batch_nnz, dtype=torch.float32, device="cuda")
    drp = torch.empty(m + 1, dtype=torch.int64, device="cuda")
    dci[:1024].copy_(ci[:1024], non_blocking=True)
    t0 = sync_time(torch)
    drp.copy_(rp, non_blocking=True)
    for e0 in range(0, nnz, batch_nnz):
        e1 = min(nnz, e0 + batch_nnz)
        dci[:e1 - e0].copy_(ci[e0:e1], non_blocking=True)
        dva[:e1 - e0].copy_(va[e0:e1], non_blocking=True)
    t1 = sync_time(torch)
    up_bytes = 8 * nnz + 8 * (m + 1)
    copy_gbs = up_bytes / (t1 - t0) / 1e9
    del dci, dva, drp
    log(f"[bench] c3ooc: CSR {m}x{n}, nnz={nnz} in pinned host memory; bare H2D copy {copy_gbs:.1f} GB/s")
    iters = args.steps
    t0 = sync_time(torch)
    nmf.nmf_mu_csr_ooc(rp, ci, va, m, n, nnz, k, W, H, iters, EPS, batch_nnz, budget)
    t1 = sync_time(torch)
    assert bool(torch.isfinite(W).all()) and bool(torch.isfinite(H).all())
    ms_step = (t1 - t0) * 1e3 / iters
    gbs = (iters + 1) * up_bytes / (t1 - t0) / 1e9
    return {"metric": "MU iterations/s (CSR fp32 streamed from pinned host memory)", "value": 1e3 / ms_step,
            "unit": "iterations/s", "n_gpus": 1, "steps": iters, "warmup": 0, "ms_per_step": ms_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"c3ooc: CSR {m}x{n}, nnz={nnz}, k={k}, batches of {batch_nnz} entries, "
                                   f"{iters} iterations = {iters + 1} uploads", "nnz": nnz},
            "h2d_gbs_achieved": gbs, "h2d_gbs_bare_copy": copy_gbs, "frac_of_bare_copy": gbs / copy_gbs}


def bench_c4(args, torch, nmf, nmf_inputs):
    m, n, k, batch = 262144, 65536, 64, 8192
    if args.small:
        m //= 8
    budget = 8 << 30
    t0 = time.perf_counter()
    Ah = torch.empty((m, n), dtype=torch.float32, pin_memory=True)
    log(f"[bench] c4: pinned {m}x{n} ({m * n * 4 / 2**30:.0f} GiB) in {time.perf_counter() - t0:.1f} s")
    t0 = time.perf_counter()
    nmf_inputs.dense_planted(m, n, 64, seed=1004, device="cuda", out=Ah, row_block=batch)
    torch.cuda.synchronize()
    log(f"[bench] c4: generated in {time.perf_counter() - t0:.1f} s")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2004, device="cuda")
    # bare copy ceiling: same chunks, same buffer, one stream
    slot = torch.empty((batch, n), dtype=torch.float32, device="cuda")
    nb = m // batch
    slot.copy_(Ah[:batch], non_blocking=True)
    t0 = sync_time(torch)
    for b in range(nb):
        slot.copy_(Ah[b * batch:(b + 1) * batch], non_blocking=True)
    t1 = sync_time(torch)
    copy_gbs = m * n * 4 / (t1 - t0) / 1e9
    del slot
    log(f"[bench] c4: bare pinned H2D copy {copy_gbs:.1f} GB/s")
    iters = args.steps
    # one short untimed call: the staging slots and the workspace are allocated by the first call
    nmf.nmf_mu_ooc(Ah[:2 * batch], 2 * batch, n, k, W[:2 * batch].clone(), H.clone(), 1, EPS, batch, budget)
    t0 = sync_time(torch)
    nmf.nmf_mu_ooc(Ah, m, n, k, W, H, iters, EPS, batch, budget)
    t1 = sync_time(torch)
    sweeps = iters + 1                     # the half-iteration skew: one upload of A more than iterations
    gbs = sweeps * m * n * 4 / (t1 - t0) / 1e9
    ms_step = (t1 - t0) * 1e3 / iters
    out = {"metric": "MU iterations/s (dense fp32, A streamed from pinned host memory)", "value": 1e3 / ms_step,
           "unit": "iterations/s", "n_gpus": 1, "steps": iters, "warmup": 0, "ms_per_step": ms_step,
           "ms_per_sweep": (t1 - t0) * 1e3 / sweeps,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"c4: dense {m}x{n} in pinned host memory, {batch}-row batches, 8 GiB staging budget, "
                                  f"k={k}, {iters} iterations = {sweeps} uploads of A"},
           "h2d_gbs_achieved": gbs, "h2d_gbs_bare_copy": copy_gbs, "frac_of_bare_copy": gbs / copy_gbs,
           # bound by the host link: achieved = bytes of A uploaded / time, peak = the bare pinned copy of the
           # same chunks measured above (PCIe Gen5 x16 is 64 GB/s raw per direction)
           "roofline": {"bound": "host link", "achieved": gbs, "peak": copy_gbs, "unit": "GB/s", "frac": gbs / copy_gbs,
                        "traffic": None, "algorithmic_bytes_per_sweep": m * n * 4}}
    if not args.no_cpu_baseline:
        from oracle import nmf_oracle as orc
        Ab = Ah[:batch].numpy()
        W0, H0 = (t.numpy() for t in nmf_inputs.init_factors(batch, n, k, seed=2004))
        t0 = time.perf_counter()
        orc.mu_dense(Ab, W0, H0, 1, EPS)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 1 / dt / (m // batch), "unit": "iterations/s", "cores": orc.num_threads(),
                               "kind": "oracle",
                               "sample": f"1 iteration on one {batch}-row batch of {m // batch} in {dt:.1f} s, scaled to the "
                                         "whole matrix (float64)"}
    return out


def bench_oom1(args, torch, nmf, nmf_inputs):
    """The paper's own out-of-memory benchmark shape (section 4.4): 524288 x 4096 fp32 (8 GiB) in 32
    row batches, A and W in pinned host memory, W_b up and down per batch (Algorithm 5), a sweep
    over the number of staging slots standing in for the stream-queue size q_s."""
    m, n, k, nbatch = 524288, 4096, args.k, 32
    if args.small:
        m //= 8
    batch = m // nbatch
    Ah = torch.empty((m, n), dtype=torch.float32, pin_memory=True)
    nmf_inputs.dense_planted(m, n, 32, seed=1006, device="cuda", out=Ah, row_block=batch)
    W0, H0 = nmf_inputs.init_factors(m, n, k, seed=2006, device="cuda")
    Wh = torch.empty((m, k), dtype=torch.float32, pin_memory=True)
    torch.cuda.synchronize()
    # bare copy ceiling of what one sweep moves up: A_b and W_b per batch, one stream
    sa = torch.empty((batch, n), dtype=torch.float32, device="cuda")
    sw = torch.empty((batch, k), dtype=torch.float32, device="cuda")
    Wh.copy_(W0)
    torch.cuda.synchronize()
    sa.copy_(Ah[:batch], non_blocking=True)
    t0 = sync_time(torch)
    for b in range(nbatch):
        sa.copy_(Ah[b * batch:(b + 1) * batch], non_blocking=True)
        sw.copy_(Wh[b * batch:(b + 1) * batch], non_blocking=True)
    t1 = sync_time(torch)
    up_bytes = m * (n + k) * 4
    copy_gbs = up_bytes / (t1 - t0) / 1e9
    del sa, sw
    log(f"[bench] oom1: {m}x{n}, k={k}, {nbatch} batches of {batch} rows; bare pinned H2D copy {copy_gbs:.1f} GB/s")
    iters = args.steps
    sweep = []
    for slots in [int(x) for x in args.slots.split(",")]:
        Wh.copy_(W0)
        H = H0.clone()
        torch.cuda.synchronize()
        t0 = sync_time(torch)
        used = nmf.nmf_mu_ooc_hostw(Ah, Wh, m, n, k, H, iters, EPS, batch, slots)
        t1 = sync_time(torch)
        assert bool(torch.isfinite(H).all()) and bool(torch.isfinite(Wh).all())
        model = min(slots, nbatch) * batch * (n + k) * 4          # the O(p n q_s) term: staged batches
        sweep.append({"slots": slots, "ms_per_iteration": (t1 - t0) * 1e3 / iters,
                      "h2d_gbs": (iters + 1) * up_bytes / (t1 - t0) / 1e9,
                      "device_bytes": used, "staged_batches_bytes": model})
        log(f"[bench] oom1: slots={slots}: {sweep[-1]}")
    best = min(sweep, key=lambda x: x["ms_per_iteration"])
    return {"metric": "MU iterations/s (dense fp32, A and W streamed from pinned host memory)",
            "value": 1e3 / best["ms_per_iteration"], "unit": "iterations/s", "n_gpus": 1, "steps": iters, "warmup": 0,
            "ms_per_step": best["ms_per_iteration"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"oom1: dense {m}x{n} and W {m}x{k} in pinned host memory, {nbatch} batches, "
                                   f"{iters} iterations = {iters + 1} sweeps, best of slots={args.slots}"},
            "h2d_gbs_achieved": best["h2d_gbs"], "h2d_gbs_bare_copy": copy_gbs,
            "frac_of_bare_copy": best["h2d_gbs"] / copy_gbs, "slot_sweep": sweep}


def bench_ck(args, torch, nmf, nmf_inputs):
    """Resident dense run at a rank above 64 (rank-sliced engine) on config 2's matrix."""
    m, n, k = 32768, 16384, args.k
    A = nmf_inputs.dense_planted(m, n, 32, seed=1002, device="cuda")
    W, H = nmf_inputs.init_factors(m, n, k, seed=2002, device="cuda")
    nmf.nmf_mu_dense(A, m, n, k, W, H, max(args.warmup, 1), EPS)
    t0 = sync_time(torch)
    nmf.nmf_mu_dense(A, m, n, k, W, H, args.steps, EPS)
    t1 = sync_time(torch)
    ms_step = (t1 - t0) * 1e3 / args.steps
    assert bool(torch.isfinite(W).all()) and bool(torch.isfinite(H).all())
    slices = (k + 63) // 64
    flop = float(flops_per_iteration(m, n, k))
    return {"metric": "MU iterations/s (dense fp32, resident A, rank-sliced)", "value": 1e3 / ms_step,
            "unit": "iterations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": f"ck: dense {m}x{n} resident, k={k} ({slices} slices of 64 factors)"},
            "gbs_over_A_reads": 2 * slices * m * n * 4 / (ms_step * 1e-3) / 1e9,
            "tflops_useful": flop / (ms_step * 1e-3) / 1e12}


def bench_c5(args, torch, nmf, nmf_inputs):
    m, n = 16384, 8192
    kmin, kmax, copies = args.kmin, args.kmax, args.copies
    base = nmf_inputs.dense_planted(m, n, 8, seed=1005, device="cuda")
    As = [nmf_inputs.perturb(base, 3000 + p) for p in range(copies)]
    runs_A, runs_k, Ws, Hs = [], [], [], []
    for p in range(copies):
        for k in range(kmin, kmax + 1):
            W, H = nmf_inputs.init_factors(m, n, k, seed=2005 + len(runs_k), device="cuda")
            runs_A.append(As[p]); runs_k.append(k); Ws.append(W); Hs.append(H)
    iters = args.steps
    nmf.nmf_mu_dense_batched(len(runs_k), runs_A, m, n, runs_k, Ws, Hs, max(args.warmup, 1), EPS)
    t0 = sync_time(torch)
    nmf.nmf_mu_dense_batched(len(runs_k), runs_A, m, n, runs_k, Ws, Hs, iters, EPS)
    t1 = sync_time(torch)
    nruns = len(runs_k)
    per_run_500 = (t1 - t0) / nruns * (500 / iters)
    useful = 4.0 * m * n * sum(runs_k) * iters              # the two products over A, fp32 multiply-adds x 2
    out = {"metric": "ensemble runs/s (500 MU iterations per run)", "value": 1.0 / per_run_500, "unit": "runs/s",
           "n_gpus": 1, "steps": iters, "warmup": args.warmup, "ms_per_step": (t1 - t0) * 1e3 / iters,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"c5: dense {m}x{n}, {copies} perturbed copies x k={kmin}..{kmax} = {nruns} runs; "
                                  f"timed {iters} iterations per run, scaled to 500"},
           "tflops_useful_fp32": useful / (t1 - t0) / 1e12,
           # matrix-core bound: every fp32 product is eight bf16 piece products, so the instructions issued
           # amount to 8 x the useful operations (stacks are padded to 32 or 64 factors on top of that)
           "roofline": {"bound": "mfma", "achieved": 8 * useful / (t1 - t0) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                        "frac": 8 * useful / (t1 - t0) / 1e12 / 2500.0, "traffic": None, "instruction": "bf16"}}
    if not args.no_cpu_baseline:
        from oracle import nmf_oracle as orc
        Ah = As[0].cpu().numpy()
        W0, H0 = (t.numpy() for t in nmf_inputs.init_factors(m, n, 8, seed=2005))
        t0 = time.perf_counter()
        orc.mu_dense(Ah, W0, H0, 2, EPS)
        dt = time.perf_counter() - t0
        # a run of rank k costs about k / 8 of this one; the ensemble's mean rank is sum(k) / runs
        scale = (sum(runs_k) / nruns) / 8.0
        out["cpu_baseline"] = {"value": 1.0 / (dt / 2 * 500 * scale), "unit": "runs/s", "cores": orc.num_threads(),
                               "kind": "oracle",
                               "sample": f"2 iterations of one k=8 run in {dt:.1f} s, scaled to 500 iterations and to the "
                                         f"ensemble's mean rank {sum(runs_k) / nruns:.1f} (float64)"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c3ooc", "c4", "c5", "oom1", "ck"])
    ap.add_argument("--k", type=int, default=128, help="rank of the oom1 / ck workloads")
    ap.add_argument("--slots", default="1,2,3,4,8", help="staging slot counts swept by oom1")
    ap.add_argument("--small", action="store_true", help="reduced c3/c4 sizes (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sub", action="store_true", help="default workload only: leave out the shortened runs of c1, c3, c4, c5")
    ap.add_argument("--calibrate", action="store_true", help="also run one plain device copy of A (counter scaling)")
    ap.add_argument("--kmin", type=int, default=2)
    ap.add_argument("--kmax", type=int, default=16)
    ap.add_argument("--copies", type=int, default=8)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import nmf_inputs
    import paper_2202_09518_amd as nmf
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    nmf.lib()   # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    fn = {"c1": bench_c1, "c2": bench_c2, "c3": bench_c3, "c3ooc": bench_c3ooc, "c4": bench_c4, "c5": bench_c5, "oom1": bench_oom1,
          "ck": bench_ck}[args.workload]
    out = fn(args, torch, nmf, nmf_inputs)
    if args.workload == "c2" and not args.no_sub:
        # The other four configurations, shortened, so that one default run times all five: same entry
        # points and launch configurations as their own --workload runs, fewer steps.
        import copy
        import gc
        out["sub_results"] = {}
        for name, steps, warm in (("c1", 200, 20), ("c3", 25, 1), ("c4", 3, 0), ("c5", 50, 1)):
            gc.collect()
            torch.cuda.synchronize()
            nmf.nmf_mu_release()
            torch.cuda.empty_cache()
            if hasattr(torch._C, "_host_emptyCache"):
                torch._C._host_emptyCache()
            a2 = copy.copy(args)
            a2.steps, a2.warmup = steps, warm
            t0 = time.perf_counter()
            r = {"c1": bench_c1, "c3": bench_c3, "c4": bench_c4, "c5": bench_c5}[name](a2, torch, nmf, nmf_inputs)
            keep = ("metric", "value", "unit", "steps", "ms_per_step", "ms_per_sweep", "config", "roofline", "cpu_baseline",
                    "gbs_over_A", "h2d_gbs_achieved", "h2d_gbs_bare_copy", "tflops_useful_fp32")
            out["sub_results"][name] = {a: r[a] for a in keep if a in r}
            out["sub_results"][name]["wall_s"] = time.perf_counter() - t0
            log(f"[bench] {name}: {r['value']:.4g} {r['unit']} ({time.perf_counter() - t0:.1f} s)")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
