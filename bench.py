#!/usr/bin/env python3
"""Benchmark of the DecentLaM hot path on one MI355X.

A "step" is one pass of the fused decentralized update (`decentlam_step`:
partial averaging + bias-corrected momentum + parameter step) over all n
simulated nodes' stacked replicas, inputs resident in HBM.  The default
workload is the headline one: n = 32 nodes, static exponential graph, d = 25.6 M
fp32 parameters per node (synthetic N(0,1) replicas and gradients).

Prints ONE JSON line.  `value` is the achieved algorithmic HBM rate of the step
(20 bytes per node-element: read x, m, g; write x, m) over wall time of K steps;
`steps_per_s` is the same measurement in steps.  `roofline` prices the step
kernel against the 8 TB/s HBM peak from HIP-event time over the same K launches;
`cpu_baseline` times the CPU oracle on a bounded column sample of the same
workload (the work is exactly linear in d).
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
BYTES_PER_ELEMENT = 20         # read x, m, g + write x, m, fp32

# HBM bytes per launch from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, each scaled by what
# the same counter reads for a plain device copy of known size), keyed by (workload, what); each entry
# names the summary under profiles/ it was read from, so that a figure can be traced (and seen to be
# stale when the kernel has changed since).  None where not measured.
MEASURED_TRAFFIC = {
    ("c3_exp32", "decentlam"): (16_383_750_981, "profiles/k_step_c3_exp32_hbm_traffic_pmc.txt"),
    ("c3_exp32", "decentlam_ld_equals_d"): (16_383_890_000,
                                            "profiles/k_step_chain_c3_exp32_ld_equals_d_kernel_stats_and_hbm_traffic.txt"),
    ("c3_exp32", "decentlam_blocked"): (16_383_742_345, "profiles/k_step_c3_exp32_layouts_tlb_and_traffic_pmc.txt"),
    ("c5_onepeer64_lsq", "local_grad_lsq"): (4_342_500_000, "profiles/local_grad_lsq_c5_hbm_traffic_pmc.txt"),
}


def measured_traffic(workload, what):
    nbytes, source = MEASURED_TRAFFIC.get((workload, what), (None, None))
    return {"traffic": nbytes, "traffic_profile": source}


def ensure_built():
    from paper_2104_11981_amd import build as hip_build

    if not os.path.exists(hip_build.LIB):
        hip_build.build()


def time_oracle_steps(w, kind, algo, d_s, target_seconds):
    """Seconds per oracle step on an n x d_s sample of the workload, with the thread count of this process."""
    import numpy as np

    import oracle

    oracle.build()
    topo = oracle.topology(kind, w.n)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((w.n, d_s))
    m = np.zeros_like(x)
    g = rng.standard_normal((w.n, d_s))
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    fn = oracle.STEP[algo]
    fn(x, m, g, topo, gamma, beta, 0)                      # warm-up (page faults, thread pool)
    t0 = time.perf_counter()
    steps = 0
    while True:
        x, m = fn(x, m, g, topo, gamma, beta, steps)
        steps += 1
        el = time.perf_counter() - t0
        if el >= target_seconds or steps >= 200:
            break
    return el / steps, steps, oracle.num_threads()


def cpu_baseline(w, kind, algo, target_seconds=12.0):
    """Time the oracle as it stands on a column sample of the same workload: with all the host cores this
    process may use, and (in a child process, since an OpenMP runtime fixes its thread count at start) with one."""
    import subprocess

    d_s = 1_280_000 if w.d >= 1_280_000 else w.d
    per_step, steps, threads = time_oracle_steps(w, kind, algo, d_s, target_seconds)
    gbs = BYTES_PER_ELEMENT * w.n * d_s / per_step / 1e9
    out = {
        "value": round(gbs, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": f"{algo} oracle (fp64 C loops, OpenMP), n={w.n}, same topology, d={d_s} columns "
                  f"({d_s / w.d:.3f} of the workload; cost is linear in d), {steps} steps, "
                  f"{per_step * 1e3:.1f} ms/step; full-size equivalent "
                  f"{1.0 / (per_step * w.d / d_s):.4f} steps/s",
        "steps_per_s_full_size_equiv": 1.0 / (per_step * w.d / d_s),
    }
    d_1 = min(d_s, 256_000)                                # one thread: a fifth of the sample, about 5 s
    env = dict(os.environ, OMP_NUM_THREADS="1")
    child = subprocess.run([sys.executable, os.path.abspath(__file__), "--oracle-one-thread", w.name, algo, str(d_1)],
                           env=env, capture_output=True, text=True)
    if child.returncode == 0 and child.stdout.strip():
        one = json.loads(child.stdout.strip().splitlines()[-1])
        out["one_thread"] = {
            "value": round(BYTES_PER_ELEMENT * w.n * d_1 / one["s_per_step"] / 1e9, 3), "unit": "GB/s", "cores": 1,
            "sample": f"the same oracle with OMP_NUM_THREADS=1 on d={d_1} columns, {one['steps']} steps, "
                      f"{one['s_per_step'] * 1e3:.1f} ms/step",
            "steps_per_s_full_size_equiv": 1.0 / (one["s_per_step"] * w.d / d_1)}
    return out


def oracle_one_thread_child(name, algo, d_s):
    import workloads

    w = workloads.get(name)
    per_step, steps, threads = time_oracle_steps(w, w.topo, algo, int(d_s), 5.0)
    print(json.dumps({"s_per_step": per_step, "steps": steps, "threads": threads}), flush=True)


def oracle_table_child():
    """Times the oracle as it stands with the OpenMP thread count this process was started with:
    every workload's step (column samples for the two large ones: the cost is linear in d) and the
    least-squares gradient of the two regression workloads.  One JSON line per row."""
    import numpy as np

    import oracle
    import workloads

    oracle.build()
    threads = oracle.num_threads()

    def timed(fn, budget=4.0, max_reps=50):
        fn()
        t0, reps = time.perf_counter(), 0
        while True:
            fn()
            reps += 1
            el = time.perf_counter() - t0
            if el >= budget or reps >= max_reps:
                return el / reps

    rng = np.random.default_rng(0)
    for name in ("c1_ring4", "c2_onepeer8_b1024", "c3_exp32", "c4_ring16_ragged", "c5_onepeer64_lsq"):
        w = workloads.get(name)
        d = workloads.generate.dim(w)
        d_s = min(d, 1_280_000)
        topo = oracle.topology(w.topo, w.n)
        x, g = rng.standard_normal((w.n, d_s)), rng.standard_normal((w.n, d_s))
        m = np.zeros_like(x)
        for algo in ("decentlam", "dmsgd"):
            sec = timed(lambda: oracle.STEP[algo](x, m, g, topo, 0.05, 0.9, 0))
            print(json.dumps({"oracle": algo + "_step", "workload": name, "threads": threads, "n": w.n, "d": d,
                              "columns_timed": d_s, "ns_per_node_element": round(sec / (w.n * d_s) * 1e9, 3),
                              "steps_per_s_full_size": round(d_s / d / sec, 4)}), flush=True)
        if w.b:
            nodes = min(w.n, 8)                     # cost is linear in the number of nodes
            A = rng.standard_normal((nodes, w.b, w.d)).astype(np.float32)
            y = rng.standard_normal((nodes, w.b)).astype(np.float32)
            xs = rng.standard_normal((nodes, w.d))
            sec = timed(lambda: oracle.lsq_grad(A, y, xs, 1.0), max_reps=10) * w.n / nodes
            print(json.dumps({"oracle": "lsq_grad", "workload": name, "threads": threads, "n": w.n, "b": w.b,
                              "d": w.d, "nodes_timed": nodes,
                              "ns_per_matrix_element": round(sec / (w.n * w.b * w.d) * 1e9, 3),
                              "calls_per_s_full_size": round(1.0 / sec, 4)}), flush=True)


def oracle_table():
    """Runs oracle_table_child with 1 thread and with all host cores (child processes: the thread
    count of an OpenMP runtime is fixed by its environment); nothing here touches the GPU."""
    import subprocess

    cores = os.cpu_count() or 1
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    for threads in (1, cores):
        env = dict(os.environ, OMP_NUM_THREADS=str(threads))
        subprocess.run([sys.executable, os.path.abspath(__file__), "--oracle-table-child"], env=env, check=True)


def time_launches(fn, steps, warmup):
    """W untimed calls, then K calls between two synchronisations; returns (wall ms, HIP-event ms) per call."""
    import torch

    for k in range(warmup):
        fn(k)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for k in range(steps):
        fn(warmup + k)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, ev0.elapsed_time(ev1) / steps


def padded_ld(d):
    """Row stride the library recommends (paper_2104_11981_amd.recommended_ld): rows start on 64 KiB
    boundaries when the arrays are large (the step then writes whole 64 KiB-aligned address pairs, see
    split tiles in step_impl.hpp; c3: 25 608 192 instead of 25 600 000 elements, +0.03 %), on 256-byte
    boundaries otherwise."""
    from paper_2104_11981_amd import recommended_ld

    return recommended_ld(d)


def all_to_all(P, n):
    """Every node averages all n with equal weights: the densest W there is."""
    import numpy as np

    return P.make_topology(n, np.arange(0, n * n + 1, n), np.tile(np.arange(n), n), np.full(n * n, 1.0 / n, np.float32))


def bench_step(P, workloads, name, algo, steps, warmup, calibration_copy=False, detail=None, ld=None, topo=None):
    import numpy as np
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    if topo is None:
        topo = P.topology_build(w.topo, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    step = getattr(P, algo + "_step")
    # Row stride: see padded_ld.  (With rows that are only 16-byte aligned every 1 KiB wave access
    # straddles an extra cache line and the ragged workload loses about 17 %: 4.65 vs 5.60 TB/s.)
    if ld is None:
        ld = padded_ld(d)
    xb = workloads.device_x0(w, "cuda", ld=ld)
    mb = torch.zeros_like(xb)
    gb = torch.zeros_like(xb)
    workloads.device_grad(w, 0, gb)
    x, m, g = xb[:, :d], mb[:, :d], gb[:, :d]
    torch.cuda.synchronize()
    # The step time settles only after about eight launches on fresh arrays (2.68, 3.25, 2.99, 2.81, 2.69, 2.62,
    # 2.60, 2.55, 2.53, 2.51 ms ... in profiles/k_step_c3_exp32_kernel_stats.txt): whatever --warmup says, at
    # least ten launches precede the timed ones, the missing ones as part of the set-up.
    for k in range(max(0, 10 - warmup)):
        step(x, m, g, topo, gamma, beta, k)
    wall_ms, kern_ms = time_launches(lambda k: step(x, m, g, topo, gamma, beta, k), steps, warmup)
    assert bool(torch.isfinite(x[:, :1024]).all()), "state overflowed during the timed run"
    if detail is not None:
        # four more repetitions of the same K-launch loop (median of five), then K launches each
        # bracketed by its own event pair with a fresh gradient generated in between
        reps = [kern_ms]
        for _ in range(4):
            xb[:, :d].normal_()
            mb.zero_()
            reps.append(time_launches(lambda k: step(x, m, g, topo, gamma, beta, k), steps, 0)[1])
        xb[:, :d].normal_()
        mb.zero_()
        fresh = []
        for k in range(steps):
            workloads.device_grad(w, k, gb)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            step(x, m, g, topo, gamma, beta, k)
            e1.record()
            torch.cuda.synchronize()
            fresh.append(e0.elapsed_time(e1))
        detail.update({"kernel_ms_repetitions": [round(v, 4) for v in reps],
                       "kernel_ms_median_of_5": round(sorted(reps)[2], 4),
                       "kernel_ms_fresh_gradient_each_launch": round(sum(fresh) / len(fresh), 4)})
    if calibration_copy:
        scratch = torch.empty_like(gb)
        scratch.copy_(gb)
        torch.cuda.synchronize()
        del scratch
    del x, m, g, xb, mb, gb
    torch.cuda.empty_cache()
    return w, d, ld, topo, wall_ms, kern_ms


def bench_xprev(P, workloads, name, steps, warmup):
    """Momentum-free DecentLaM (state x^k, x^{k-1}; 16 bytes per node-element), buffers rotated per step."""
    import numpy as np
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    topo = P.topology_build(w.topo, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    full = [workloads.device_x0(w, "cuda", ld=padded_ld(d))]
    full.append(full[0].clone())
    gb = torch.zeros_like(full[0])
    workloads.device_grad(w, 0, gb)
    bufs, g = [b[:, :d] for b in full], gb[:, :d]
    torch.cuda.synchronize()

    def step(k):
        P.decentlam_step_xprev(bufs[k % 2], bufs[(k + 1) % 2], g, topo, gamma, beta, k)

    _, kern_ms = time_launches(step, steps, warmup)
    nbytes = 16 * w.n * d
    del bufs, g, full, gb
    torch.cuda.empty_cache()
    return {"kernel_ms": round(kern_ms, 4), "bytes_per_node_element": 16,
            "GBps": round(nbytes / (kern_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "steps_per_s": round(1e3 / kern_ms, 1)}


HEADLINE_ELEMENTS = 32 * 25_600_000


def bench_shape(P, n, d, kind, steps, warmup):
    """decentlam_step on a synthetic n x d state with a built-in graph (values N(0,1), zero momentum)."""
    import torch

    topo = P.topology_build(kind, n)
    x, m, g = (P.empty_rows(n, d) for _ in range(3))
    x.normal_()
    m.zero_()
    g.normal_()
    _, ms = time_launches(lambda k: P.decentlam_step(x, m, g, topo, 0.01, 0.9, k), steps, warmup)
    nbytes = BYTES_PER_ELEMENT * n * d
    del x, m, g
    torch.cuda.empty_cache()
    return {"n": n, "d": d, "kernel_ms": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "steps_per_s": round(1e3 / ms, 1)}


def bench_copy(P, workloads, name, steps, warmup):
    """What this GPU gives a plain device-to-device copy of one n x ld fp32 array of the workload (torch's
    copy_: reads and writes 4 * n * ld bytes), as context for the roofline fractions."""
    import torch

    w = workloads.get(name)
    ld = padded_ld(workloads.generate.dim(w))
    src = torch.zeros((w.n, ld), dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    _, ms = time_launches(lambda k: dst.copy_(src), steps, warmup)
    nbytes = 2.0 * 4.0 * w.n * ld
    del src, dst
    torch.cuda.empty_cache()
    return {"ms": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def bench_stream(P, workloads, name, steps, warmup, ld=None):
    """The achievable-bandwidth denominator: bare streams with the step kernel's access pattern
    (dl_calibration_stream: same tiles, same 16-byte non-temporal accesses, no arithmetic of the method) on
    arrays of the workload's shape, in the column order of the step's large launches."""
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    if ld is None:
        ld = padded_ld(d)
    bufs = [torch.zeros((w.n, ld), dtype=torch.float32, device="cuda") for _ in range(3)]
    bufs[0].normal_()
    bufs[2].normal_()
    x, m, g = (b[:, :d] for b in bufs)
    out = {"ld": ld}
    for key, kind, nbytes in (("stream_3r2w", 0, 20), ("stream_read", 1, 12), ("stream_write", 2, 8)):
        cols = P.dl_calibration_stream(kind, True, x, m, g)
        _, ms = time_launches(lambda k: P.dl_calibration_stream(kind, True, x, m, g), steps, warmup)
        out[key + "_ms"] = round(ms, 4)
        out[key + "_GBps"] = round(nbytes * w.n * cols / (ms * 1e-3) / 1e9, 1)
    out["columns_covered"] = cols
    del x, m, g, bufs
    torch.cuda.empty_cache()
    return out


def bench_stats(P, workloads, name, steps, warmup):
    """decentlam_stats (consensus distance, mean norm, error against a reference, momentum norm) on the
    workload's state: one pass over x and m, 8 bytes per node-element plus the reference vector."""
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    ld = padded_ld(d)
    xb = workloads.device_x0(w, "cuda", ld=ld)
    mb = torch.zeros_like(xb)
    workloads.device_grad(w, 0, mb)
    x, m = xb[:, :d], mb[:, :d]
    ref = torch.zeros(d, dtype=torch.float32, device="cuda")
    out = torch.empty(5, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_stats_workspace(w.n, d), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    _, kern_ms = time_launches(lambda k: P.decentlam_stats(x, m, ref, out, ws), steps, warmup)
    nbytes = 8 * w.n * d + 4 * d
    del x, m, xb, mb, ref
    torch.cuda.empty_cache()
    return {"ms_per_call": round(kern_ms, 4), "GBps": round(nbytes / (kern_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def bench_blocked(P, workloads, name, algo, steps, warmup, bw=8192, calibration_copy=False):
    """The same n x d step on arrays in the blocked layout (blocks of bw columns, each a row-major
    n x bw matrix): the n rows a workgroup touches lie within n*bw*4 bytes instead of being d*4 bytes
    apart."""
    import numpy as np
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    nb = (d + bw - 1) // bw
    topo = P.topology_build(w.topo, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    gen = torch.Generator(device="cuda").manual_seed(workloads.BASE_SEED % (2 ** 31))
    x = torch.empty((nb, w.n, bw), dtype=torch.float32, device="cuda").normal_(generator=gen)
    m = torch.zeros_like(x)
    g = torch.empty_like(x).normal_(generator=gen)
    step = getattr(P, algo + "_step_blocked")
    wall_ms, kern_ms = time_launches(lambda k: step(x, m, g, d, topo, gamma, beta, k), steps, warmup)
    assert bool(torch.isfinite(x[0, :, :1024]).all()), "state overflowed during the timed run"
    nbytes = BYTES_PER_ELEMENT * w.n * d
    if calibration_copy:
        scratch = torch.empty_like(g)
        scratch.copy_(g)
        torch.cuda.synchronize()
        del scratch
    del x, m, g
    torch.cuda.empty_cache()
    return {"kernel_ms": round(kern_ms, 4), "wall_ms": round(wall_ms, 4), "block_columns": bw,
            "GBps": round(nbytes / (kern_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "steps_per_s": round(1e3 / wall_ms, 1)}


def bench_lean(P, workloads, name, steps, warmup, bw=8192):
    """The leanest iteration on offer: momentum-free DecentLaM (state x^k, x^{k-1}), bf16 gradients,
    blocked layout: 14 bytes per node-element."""
    import numpy as np
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    nb = (d + bw - 1) // bw
    topo = P.topology_build(w.topo, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    gen = torch.Generator(device="cuda").manual_seed(workloads.BASE_SEED % (2 ** 31))
    bufs = [torch.empty((nb, w.n, bw), dtype=torch.float32, device="cuda").normal_(generator=gen)]
    bufs.append(bufs[0].clone())
    g = torch.empty((nb, w.n, bw), dtype=torch.float32, device="cuda").normal_(generator=gen).to(torch.bfloat16)

    def step(k):
        P.decentlam_step_xprev_ex(bufs[k % 2], bufs[(k + 1) % 2], g, topo, gamma, beta, k, d=d)

    _, kern_ms = time_launches(step, steps, warmup)
    nbytes = 14 * w.n * d
    del bufs, g
    torch.cuda.empty_cache()
    return {"kernel_ms": round(kern_ms, 4), "bytes_per_node_element": 14, "block_columns": bw,
            "GBps": round(nbytes / (kern_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "steps_per_s": round(1e3 / kern_ms, 1)}


def bench_g16(P, workloads, name, steps, warmup, dtype_name="bfloat16"):
    """DecentLaM step with 16-bit gradients (x, m fp32): 18 bytes per node-element."""
    import numpy as np
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    topo = P.topology_build(w.topo, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    ld = padded_ld(d)
    xb = workloads.device_x0(w, "cuda", ld=ld)
    mb = torch.zeros_like(xb)
    g32 = torch.zeros_like(xb)
    workloads.device_grad(w, 0, g32)
    gb = g32.to(getattr(torch, dtype_name))
    del g32
    x, m, g = xb[:, :d], mb[:, :d], gb[:, :d]
    _, kern_ms = time_launches(lambda k: P.decentlam_step_g16(x, m, g, topo, gamma, beta, k), steps, warmup)
    nbytes = 18 * w.n * d
    del x, m, g, xb, mb, gb
    torch.cuda.empty_cache()
    return {"kernel_ms": round(kern_ms, 4), "bytes_per_node_element": 18, "g_format": dtype_name,
            "GBps": round(nbytes / (kern_ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "steps_per_s": round(1e3 / kern_ms, 1)}


def bench_multi(P, workloads, name, steps, warmup):
    """Ragged workload as one multi-tensor call with per-tensor sums of squares of g, m, x
    (table upload + fused step + final per-tensor pass), timed as a whole."""
    import numpy as np
    import torch

    w = workloads.get(name)
    d = workloads.generate.dim(w)
    _, offsets, _ = workloads.ragged_layout(w)
    offsets = np.asarray(offsets, dtype=np.int64)
    topo = P.topology_build(w.topo, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    ld = padded_ld(d)
    x = workloads.device_x0(w, "cuda", ld=ld)
    m = torch.zeros_like(x)
    g = torch.zeros_like(x)
    workloads.device_grad(w, 0, g)
    T = offsets.size - 1
    norms = torch.empty((T, w.n, 3), dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_step_multi_workspace(w.n, d, T) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    _, ms = time_launches(lambda k: P.decentlam_step_multi(x, m, g, offsets, topo, gamma, beta, k,
                                                           norms=norms, workspace=ws), steps, warmup)
    nbytes = BYTES_PER_ELEMENT * w.n * d
    del x, m, g, ws, norms
    torch.cuda.empty_cache()
    return {"ms_per_call": round(ms, 4), "tensors": int(T), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def bench_graph(P, workloads, name, replays=200):
    """Launch-bound small workload: one period of the time-varying topology (gradient + DecentLaM step
    per iteration) captured once in a HIP graph and replayed; microseconds per iteration, eager beside it."""
    import numpy as np
    import torch

    w = workloads.get(name)
    A, y, _ = workloads.device_lsq_problem(w, "cuda")
    topo = P.topology_build(w.topo, w.n)
    gamma, beta, scale = (float(np.float32(v)) for v in (w.gamma, w.beta, w.lsq_scale))
    x = torch.zeros((w.n, w.d), dtype=torch.float32, device="cuda")
    m, g = torch.zeros_like(x), torch.zeros_like(x)
    ws = torch.empty(P.local_grad_lsq_workspace(w.n, w.b, w.d), dtype=torch.uint8, device="cuda")

    def period():
        for k in range(topo.period):
            P.local_grad_lsq(A, y, x, g, None, scale, ws)
            P.decentlam_step(x, m, g, topo, gamma, beta, k)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        period()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        period()
    x.zero_()
    m.zero_()
    _, graph_ms = time_launches(lambda k: graph.replay(), replays, 5)
    x.zero_()
    m.zero_()
    _, eager_ms = time_launches(lambda k: period(), replays, 5)
    return {"iterations_per_graph": topo.period, "graph_us_per_iteration": round(graph_ms * 1e3 / topo.period, 2),
            "eager_us_per_iteration": round(eager_ms * 1e3 / topo.period, 2)}


def bench_small(P, workloads, steps=2000, warmup=200):
    """The launch-latency-bound workloads with W packed once (topology_pack) and the calls' arguments marshalled
    once (prepare_step, prepare_local_grad_lsq): microseconds per iteration of workload 1 (one step) and of
    workload 2 with b = 32 (gradient, then step), eager launches on one stream."""
    import numpy as np
    import torch

    out = {}
    w = workloads.get("c1_ring4")
    packed = P.topology_pack(P.topology_build(w.topo, w.n))
    x = workloads.device_x0(w, "cuda", ld=w.d)
    m, g = torch.zeros_like(x), torch.zeros_like(x)
    workloads.device_grad(w, 0, g)
    step = P.prepare_step("decentlam", x, m, g, packed, 1e-3, float(np.float32(w.beta)))
    _, ms = time_launches(step, steps, warmup)
    out["c1_ring4_step_us"] = round(ms * 1e3, 2)
    w = workloads.get("c2_onepeer8_b32")
    A, y, _ = workloads.device_lsq_problem(w, "cuda")
    packed = P.topology_pack(P.topology_build(w.topo, w.n))
    gamma, beta, scale = (float(np.float32(v)) for v in (w.gamma, w.beta, w.lsq_scale))
    x = torch.zeros((w.n, w.d), dtype=torch.float32, device="cuda")
    m, g = torch.zeros_like(x), torch.zeros_like(x)
    ws = torch.empty(P.local_grad_lsq_workspace(w.n, w.b, w.d), dtype=torch.uint8, device="cuda")
    grad = P.prepare_local_grad_lsq(A, y, x, g, None, scale, ws)
    step = P.prepare_step("dmsgd", x, m, g, packed, gamma, beta)   # DmSGD: this workload's DecentLaM run diverges

    def iteration(k):
        grad()
        step(k)

    _, ms = time_launches(iteration, steps, warmup)
    out["c2_onepeer8_b32_grad_plus_step_us"] = round(ms * 1e3, 2)
    _, ms = time_launches(lambda k: grad(), steps, warmup)
    out["c2_onepeer8_b32_grad_us"] = round(ms * 1e3, 2)
    return out


def bench_lsq_shape(P, n, b, d, steps, warmup, sampled=0):
    """local_grad_lsq on synthetic N(0,1) data of the given shape: time per call, rate of the 4 n b d bytes of A.
    sampled > 0: the mini-batch form over that many of the b rows per node, drawn at random without replacement
    (seeded); the rate is then that of the rows read."""
    import torch

    A = torch.randn((n, b, d), device="cuda")
    y = torch.randn((n, b), device="cuda")
    x = torch.randn((n, d), device="cuda")
    g = torch.empty_like(x)
    rows = None
    if sampled:
        gen = torch.Generator(device="cuda").manual_seed(11981)
        rows = torch.stack([torch.randperm(b, device="cuda", generator=gen)[:sampled] for _ in range(n)]).to(torch.int32).contiguous()
    ws = torch.empty(P.local_grad_lsq_workspace(n, sampled or b, d), dtype=torch.uint8, device="cuda")
    _, ms = time_launches(lambda k: P.local_grad_lsq(A, y, x, g, None, 1.0, ws, rows=rows), steps, warmup)
    nbytes = 4 * n * (sampled or b) * d
    del A, y, x, g, ws
    torch.cuda.empty_cache()
    return {"ms_per_call": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}


def bench_lsq(P, workloads, name, steps, warmup, calibration_copy=False):
    """Workload 5: local_grad_lsq then decentlam_step per iteration; times the gradient alone too."""
    import numpy as np
    import torch

    w = workloads.get(name)
    A, y, _ = workloads.device_lsq_problem(w, "cuda")
    topo = P.topology_build(w.topo, w.n)
    gamma, beta, scale = (float(np.float32(v)) for v in (w.gamma, w.beta, w.lsq_scale))
    x = torch.zeros((w.n, w.d), dtype=torch.float32, device="cuda")
    m = torch.zeros_like(x)
    g = torch.empty_like(x)
    loss = torch.empty(w.n, dtype=torch.float32, device="cuda")
    ws = torch.empty(P.local_grad_lsq_workspace(w.n, w.b, w.d), dtype=torch.uint8, device="cuda")

    def iteration(k):
        P.local_grad_lsq(A, y, x, g, loss, scale, ws)
        P.decentlam_step(x, m, g, topo, gamma, beta, k)

    wall_ms, both_ms = time_launches(iteration, steps, warmup)
    _, grad_ms = time_launches(lambda k: P.local_grad_lsq(A, y, x, g, loss, scale, ws), steps, 1)
    a_bytes = 4 * w.n * w.b * w.d
    if calibration_copy:
        scratch = torch.empty_like(A)
        scratch.copy_(A)
        torch.cuda.synchronize()
        del scratch
    del A, y, x, m, g, ws
    torch.cuda.empty_cache()
    return {
        "workload": w.name, "n": w.n, "b": w.b, "d": w.d,
        "ms_per_iteration_grad_plus_step": round(wall_ms, 4), "grad_kernel_ms": round(grad_ms, 4),
        "grad_algorithmic_bytes": a_bytes, "grad_GBps": round(a_bytes / (grad_ms * 1e-3) / 1e9, 1),
        "grad_frac_of_hbm_peak": round(a_bytes / (grad_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "grad_GFLOPps_fp64": round(4.0 * w.n * w.b * w.d / (grad_ms * 1e-3) / 1e9, 1),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10,
                    help="untimed launches before the timed ones (the step time settles after about eight launches)")
    ap.add_argument("--workload", default="c3_exp32",
                    choices=["c3_exp32", "c4_ring16_ragged", "c5_onepeer64_lsq"])
    ap.add_argument("--algo", default="decentlam", choices=["decentlam", "dmsgd"])
    ap.add_argument("--layout", default="rowmajor", choices=["rowmajor", "blocked"],
                    help="rowmajor: decentlam_step / dmsgd_step on n x d arrays with row stride ld (the default); "
                         "blocked: the *_step_blocked calls on the same problem stored in blocks of "
                         "--block-columns columns")
    ap.add_argument("--ld", default="padded", choices=["padded", "d"],
                    help="row stride of the row-major line: 'padded' = rows on 64 KiB boundaries (what the header "
                         "recommends; +0.03 %% of memory on the headline workload), 'd' = no padding at all")
    ap.add_argument("--block-columns", type=int, default=8192)
    ap.add_argument("--all-to-all", action="store_true",
                    help="row-major line only: replace the workload's graph by all-to-all averaging with equal "
                         "weights (the mixing then runs on the matrix cores; a side measurement, not the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the side measurements (DmSGD, ragged workload, least-squares gradient)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, run one plain device copy of one n x d array "
                         "(known size: reads and writes 4*n*d bytes) so that a rocprofv3 --pmc run "
                         "of this command can scale FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--streams-only", action="store_true",
                    help="only the bare calibration streams (dl_calibration_stream) on the workload's shape, with "
                         "rows padded to 64 KiB boundaries and with ld = d: one JSON line (used for the profiles)")
    ap.add_argument("--node-counts", default=None, metavar="N1,N2,...",
                    help="only decentlam_step at these node counts on arrays of the headline size (819.2 M node-elements, "
                         "rows on 64 KiB boundaries), ring and static exponential graph: one JSON line (used for the "
                         "profiles)")
    ap.add_argument("--lsq-shapes", default=None, metavar="N:B:D,...",
                    help="only local_grad_lsq on synthetic problems of these shapes (n nodes of b x d): one JSON line "
                         "(used for the profiles)")
    ap.add_argument("--oracle-table", action="store_true",
                    help="CPU only: time the oracle on every workload at 1 thread and at all host cores")
    ap.add_argument("--oracle-table-child", action="store_true", help=argparse.SUPPRESS)
    ap.add_argument("--oracle-one-thread", nargs=3, metavar=("WORKLOAD", "ALGO", "COLUMNS"), help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.oracle_one_thread:
        oracle_one_thread_child(*args.oracle_one_thread)
        return
    if args.oracle_table_child:
        oracle_table_child()
        return
    if args.oracle_table:
        oracle_table()
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build simulates all n nodes on ONE GPU (columns of the update are "
                 "independent, so sharding d over GPUs needs no exchange); run with --gpus 1")
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: single-process benchmark; do not launch it under torch.distributed.run")

    ensure_built()
    import torch

    import paper_2104_11981_amd as P
    import workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)

    if args.node_counts:
        out = {}
        for n in (int(v) for v in args.node_counts.split(",")):
            for kind, name in ((P.DL_TOPO_RING, "ring"), (P.DL_TOPO_EXP_STATIC, "exp_static")):
                out[f"n{n}_{name}"] = bench_shape(P, n, HEADLINE_ELEMENTS // n, kind, args.steps, args.warmup)
        if args.calibration_copy:   # one plain device copy of 819.2 M floats: what the counters read for a known size
            a = torch.empty(HEADLINE_ELEMENTS, dtype=torch.float32, device="cuda").normal_()
            b = torch.empty_like(a)
            b.copy_(a)
            torch.cuda.synchronize()
            del a, b
        print(json.dumps({"what": "decentlam_step by node count, 819.2 M node-elements, rows on 64 KiB boundaries",
                          "steps": args.steps, "warmup": args.warmup, **out}), flush=True)
        return
    if args.lsq_shapes:
        out = {}
        for n, b, d in (tuple(int(v) for v in shape.split(":")) for shape in args.lsq_shapes.split(",")):
            out[f"n{n}_b{b}_d{d}"] = bench_lsq_shape(P, n, b, d, args.steps, args.warmup)
        if args.calibration_copy:   # one plain device copy of 2^29 floats: what the counters read for a known size
            a = torch.empty(1 << 29, dtype=torch.float32, device="cuda").normal_()
            b = torch.empty_like(a)
            b.copy_(a)
            torch.cuda.synchronize()
            del a, b
        print(json.dumps({"what": "local_grad_lsq by shape, rate of the 4 n b d bytes of A", "steps": args.steps,
                          "warmup": args.warmup, **out}), flush=True)
        return
    if args.streams_only:
        d0 = workloads.generate.dim(workloads.get(args.workload))
        print(json.dumps({"workload": args.workload, "steps": args.steps, "warmup": args.warmup,
                          "rows_on_64KiB": bench_stream(P, workloads, args.workload, args.steps, args.warmup),
                          "ld_equals_d": bench_stream(P, workloads, args.workload, args.steps, args.warmup, ld=d0)}),
              flush=True)
        return
    if args.workload == "c5_onepeer64_lsq":
        # side workload: one iteration = local_grad_lsq + decentlam_step; the gradient kernel dominates
        r = bench_lsq(P, workloads, args.workload, args.steps, args.warmup, args.calibration_copy)
        print(json.dumps({
            "metric": "least-squares workload: local_grad_lsq + decentlam_step per iteration (n=64, A_i 4096x4096)",
            "value": round(r["grad_algorithmic_bytes"] / (r["ms_per_iteration_grad_plus_step"] * 1e-3) / 1e9, 2),
            "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": r["ms_per_iteration_grad_plus_step"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": args.workload, "n": r["n"], "b": r["b"], "d": r["d"]},
            "roofline": {"bound": "hbm", "achieved": r["grad_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": r["grad_frac_of_hbm_peak"],
                         **measured_traffic(args.workload, "local_grad_lsq"),
                         "kernel": "k_fused", "kernel_ms": r["grad_kernel_ms"],
                         "algorithmic_bytes_per_launch": r["grad_algorithmic_bytes"]},
        }), flush=True)
        return
    if args.layout == "blocked":
        # the same problem in the blocked layout, as a line of its own (used for the profiles)
        w = workloads.get(args.workload)
        d = workloads.generate.dim(w)
        r = bench_blocked(P, workloads, args.workload, args.algo, args.steps, args.warmup, args.block_columns,
                          args.calibration_copy)
        nbytes = BYTES_PER_ELEMENT * w.n * d
        print(json.dumps({
            "metric": f"{args.algo} step, blocked layout: achieved HBM GB/s & steps/s ({w.name})",
            "value": round(nbytes / (r["wall_ms"] * 1e-3) / 1e9, 2), "unit": "GB/s", "steps_per_s": r["steps_per_s"],
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["wall_ms"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": w.name, "algo": args.algo, "n": w.n, "d": d, "layout": "blocked",
                       "block_columns": args.block_columns, "bytes_per_node_element": BYTES_PER_ELEMENT},
            "roofline": {"bound": "hbm", "achieved": r["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": r["frac_of_hbm_peak"],
                         **measured_traffic(args.workload, args.algo + "_blocked"),
                         "kernel": "k_step", "kernel_ms": r["kernel_ms"], "algorithmic_bytes_per_launch": nbytes},
        }), flush=True)
        return
    detail = None if args.no_extras else {}
    w, d, ld, topo, wall_ms, kern_ms = bench_step(
        P, workloads, args.workload, args.algo, args.steps, args.warmup, args.calibration_copy, detail,
        ld=workloads.generate.dim(workloads.get(args.workload)) if args.ld == "d" else None,
        topo=all_to_all(P, workloads.get(args.workload).n) if args.all_to_all else None)
    kind = w.topo
    bytes_per_step = BYTES_PER_ELEMENT * w.n * d
    value = bytes_per_step / (wall_ms * 1e-3) / 1e9
    achieved = bytes_per_step / (kern_ms * 1e-3) / 1e9

    out = {
        "metric": "DecentLaM step: achieved HBM GB/s & steps/s at n=32 nodes x d=25.6M fp32"
        if (args.workload, args.algo, args.all_to_all) == ("c3_exp32", "decentlam", False)
        else f"{args.algo} step: achieved HBM GB/s & steps/s ({w.name}{', all-to-all graph' if args.all_to_all else ''})",
        "value": round(value, 2), "unit": "GB/s",
        "steps_per_s": round(1e3 / wall_ms, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": w.name, "algo": args.algo, "n": w.n, "d": d, "ld": ld,
                   "layout": "row-major, ld = d (no padding)" if ld == d else
                             "row-major, rows padded to 64 KiB boundaries (ld = %d, +%.2f %% of memory)" % (ld, 100.0 * (ld - d) / d),
                   "topology": "all_to_all" if args.all_to_all else {0: "ring", 1: "exp_static", 2: "exp_onepeer"}[kind],
                   "deg": int(topo.row_ptr[1] - topo.row_ptr[0]), "gamma": w.gamma, "beta": w.beta,
                   "storage": "fp32", "bytes_per_node_element": BYTES_PER_ELEMENT},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     **(measured_traffic(args.workload, args.algo + ("_ld_equals_d" if args.ld == "d" else ""))
                        if not args.all_to_all else {"traffic": None, "traffic_profile": None}),
                     "kernel": "k_step_chain" if (args.ld == "d" and args.workload == "c3_exp32" and not args.all_to_all)
                     else "k_step", "kernel_ms": round(kern_ms, 4),
                     "algorithmic_bytes_per_launch": bytes_per_step},
    }
    if args.all_to_all:
        out["mix_fp64_mfma_TFLOPps"] = round(2.0 * w.n * w.n * d / (kern_ms * 1e-3) / 1e12, 2)
    if not args.no_extras:
        extras = dict(detail)
        for name, algo in (("c3_exp32", "dmsgd"), ("c4_ring16_ragged", "decentlam"), ("c3_exp32", "awc_dmsgd"),
                           ("c3_exp32", "da_dmsgd")):
            if (name, algo) == (args.workload, args.algo):
                continue
            w2, d2, _, _, _, k2 = bench_step(P, workloads, name, algo, args.steps, args.warmup)
            b2 = BYTES_PER_ELEMENT * w2.n * d2
            extras[f"{algo}_step_{name}"] = {"kernel_ms": round(k2, 4), "steps_per_s": round(1e3 / k2, 1),
                                             "GBps": round(b2 / (k2 * 1e-3) / 1e9, 1),
                                             "frac_of_hbm_peak": round(b2 / (k2 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        w3 = workloads.get("c3_exp32")
        d3 = workloads.generate.dim(w3)
        b3 = BYTES_PER_ELEMENT * w3.n * d3
        # c3 with no padding at all (ld = d = 3125 x 32 KiB: odd rows start in the upper half of a
        # 64 KiB unit, so only every other row can write whole address pairs)
        _, _, _, _, _, k4 = bench_step(P, workloads, "c3_exp32", "decentlam", args.steps, args.warmup, ld=d3)
        extras["decentlam_step_c3_exp32_ld_equals_d"] = {
            "kernel_ms": round(k4, 4), "steps_per_s": round(1e3 / k4, 1), "GBps": round(b3 / (k4 * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(b3 / (k4 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        if (args.workload, args.algo, args.ld, args.all_to_all) == ("c3_exp32", "decentlam", "padded", False):
            # the same workload with the row stride the workload states (a contiguous 32 x 25.6 M array): the
            # headline beside it is measured on rows padded to 64 KiB boundaries, which the header recommends
            out["roofline_ld_equals_d"] = {
                "bound": "hbm", "achieved": round(b3 / (k4 * 1e-3) / 1e9, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(b3 / (k4 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                **measured_traffic("c3_exp32", "decentlam_ld_equals_d"), "kernel": "k_step_chain",
                "kernel_ms": round(k4, 4), "steps_per_s": round(1e3 / k4, 1), "ld": d3,
                "algorithmic_bytes_per_launch": b3}
        # c3's arrays under all-to-all averaging (1024 entries): the mixing runs as an fp64 product on
        # the matrix cores, 2 n^2 d flops per step beside the same 20 B per node-element
        _, _, _, _, _, k5 = bench_step(P, workloads, "c3_exp32", "decentlam", args.steps, args.warmup,
                                       topo=all_to_all(P, w3.n))
        extras["decentlam_step_c3_all_to_all32"] = {
            "kernel_ms": round(k5, 4), "GBps": round(b3 / (k5 * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(b3 / (k5 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "mix_fp64_mfma_TFLOPps": round(2.0 * w3.n * w3.n * d3 / (k5 * 1e-3) / 1e12, 2)}
        extras["decentlam_step_xprev_c3_exp32"] = bench_xprev(P, workloads, "c3_exp32", args.steps, args.warmup)
        blk = bench_blocked(P, workloads, "c3_exp32", "decentlam", args.steps, args.warmup)
        extras["decentlam_step_blocked_c3_exp32"] = blk
        if (args.workload, args.algo) == ("c3_exp32", "decentlam"):
            # the same workload through decentlam_step_blocked (arrays stored in blocks of 8192 columns):
            # same arithmetic, same bytes
            out["roofline_blocked_layout"] = {
                "bound": "hbm", "achieved": blk["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": blk["frac_of_hbm_peak"], **measured_traffic("c3_exp32", "decentlam_blocked"),
                "kernel": "k_step", "kernel_ms": blk["kernel_ms"], "steps_per_s": blk["steps_per_s"],
                "algorithmic_bytes_per_launch": bytes_per_step, "entry_point": "decentlam_step_blocked",
                "block_columns": blk["block_columns"]}
        extras["dmsgd_step_blocked_c3_exp32"] = bench_blocked(P, workloads, "c3_exp32", "dmsgd", args.steps,
                                                              args.warmup)
        extras["decentlam_step_xprev_bf16_blocked_c3_exp32"] = bench_lean(P, workloads, "c3_exp32", args.steps,
                                                                          args.warmup)
        extras["decentlam_step_g16_bf16_c3_exp32"] = bench_g16(P, workloads, "c3_exp32", args.steps, args.warmup)
        extras["decentlam_step_multi_norms_c4_ring16_ragged"] = bench_multi(P, workloads, "c4_ring16_ragged",
                                                                             args.steps, args.warmup)
        # the paper's own scale: 8 nodes (its servers), symmetric exponential graph, a ResNet-50-sized vector
        # other node counts on arrays of the headline size (the kernel and its workgroup shape change with n)
        extras["decentlam_step_by_node_count_exp_static"] = {
            f"n{n}": bench_shape(P, n, HEADLINE_ELEMENTS // n, P.DL_TOPO_EXP_STATIC, args.steps, args.warmup)
            for n in (16, 48, 64, 128)}
        extras["decentlam_step_8_nodes_sym_exp_25.6M"] = bench_shape(P, 8, 25_600_000, P.DL_TOPO_EXP_SYM,
                                                                    args.steps, args.warmup)
        extras["plain_device_copy_c3_array"] = bench_copy(P, workloads, "c3_exp32", args.steps, args.warmup)
        # what the memory gives bare streams with the step's access pattern on c3-shaped arrays (both row strides)
        st = bench_stream(P, workloads, "c3_exp32", args.steps, args.warmup)
        extras["calibration_streams_c3_shape"] = st
        extras["calibration_streams_c3_shape_ld_equals_d"] = bench_stream(P, workloads, "c3_exp32", args.steps,
                                                                           args.warmup, ld=d3)
        if (args.workload, args.ld, args.all_to_all) == ("c3_exp32", "padded", False):
            out["stream_3r2w_GBps"] = st["stream_3r2w_GBps"]
            out["stream_read_GBps"] = st["stream_read_GBps"]
            out["stream_write_GBps"] = st["stream_write_GBps"]
            out["roofline"]["frac_of_measured_stream"] = round(achieved / st["stream_3r2w_GBps"], 4)
        extras["decentlam_stats_c3_exp32"] = bench_stats(P, workloads, "c3_exp32", args.steps, args.warmup)
        c5 = bench_lsq(P, workloads, "c5_onepeer64_lsq", args.steps, args.warmup)
        extras["local_grad_lsq_c5"] = c5
        # rows too wide for the register-resident x_i (16384 < d <= 32768: the widest form of a workgroup per row tile),
        # wider still (up to 262144: the columns of a row split over waves, still one sweep) and beyond (two sweeps)
        extras["local_grad_lsq_wide_rows"] = {
            f"n{n}_b{b}_d{d}": bench_lsq_shape(P, n, b, d, args.steps, args.warmup)
            for n, b, d in ((8, 2048, 32768), (8, 1024, 65536), (4, 1024, 131072), (2, 1024, 262144), (1, 1024, 524288))}
        # short rows: a wave per row (or per two rows)
        extras["local_grad_lsq_short_rows"] = {
            f"n{n}_b{b}_d{d}": bench_lsq_shape(P, n, b, d, args.steps, args.warmup)
            for n, b, d in ((64, 4096, 1024), (64, 32768, 128))}
        # the mini-batch form: rows drawn at random from each node's 4096
        extras["local_grad_lsq_sampled_rows"] = {
            f"n64_b4096_d4096_bs{bs}": bench_lsq_shape(P, 64, 4096, 4096, args.steps, args.warmup, sampled=bs)
            for bs in (1024, 4096)}
        # contiguous A whose rows are not on 16-byte boundaries: on 8-byte ones (even d) and on none (odd d)
        extras["local_grad_lsq_rows_off_16_byte_boundaries"] = {
            f"n{n}_b{b}_d{d}": bench_lsq_shape(P, n, b, d, args.steps, args.warmup)
            for n, b, d in ((8, 4096, 7850), (16, 4096, 4095))}
        # the two other large workloads under their own names: iterations per second and fraction of the HBM peak
        c4 = extras.get("decentlam_step_c4_ring16_ragged")
        if c4:
            out["c4_ring16_ragged"] = {"steps_per_s": c4["steps_per_s"], "GBps": c4["GBps"], "frac": c4["frac_of_hbm_peak"],
                                       "what": "decentlam_step, one flat call over the 160 packed tensors, 20 B per node-element"}
        out["c5_onepeer64_lsq"] = {
            "steps_per_s": round(1e3 / c5["ms_per_iteration_grad_plus_step"], 1),
            "grad_GBps": c5["grad_GBps"], "frac": c5["grad_frac_of_hbm_peak"],
            "what": "local_grad_lsq + decentlam_step per iteration; frac prices the gradient call against 4 n b d bytes"}
        # the small least-squares workloads are cache-resident and latency-bound: microseconds only
        for small in ("c2_onepeer8_b32", "c2_onepeer8_b1024"):
            r2 = bench_lsq(P, workloads, small, 200, 20)
            extras[f"{small}_us"] = {"grad_plus_step": round(r2["ms_per_iteration_grad_plus_step"] * 1e3, 2),
                                     "grad": round(r2["grad_kernel_ms"] * 1e3, 2)}
        extras["c2_onepeer8_b32_hip_graph"] = bench_graph(P, workloads, "c2_onepeer8_b32")
        # the small workloads are launch-latency bound: report microseconds per call
        w1 = workloads.get("c1_ring4")
        _, _, _, _, _, k1 = bench_step(P, workloads, "c1_ring4", "decentlam", 200, 20)
        extras["decentlam_step_c1_ring4_us"] = round(k1 * 1e3, 2)
        # the same small workloads with W packed once and the calls' arguments marshalled once
        extras["small_workloads_prepared_calls"] = bench_small(P, workloads)
        out["extras"] = extras
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, kind, args.algo)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
