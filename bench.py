#!/usr/bin/env python3
"""Benchmark of the elastic AdaHessian hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input: dw_worker_step for all k workers
(forward, backward, Hessian-vector product, fused AdaHessian update) followed by dw_elastic_sync, which
takes a communication round every tau steps.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line: metric/value (worker-steps/s over the whole job), a `roofline` object for the kernel
class that takes the most time (HIP-event timing of every launch in a second pass over the same steps), a
`kernels` breakdown, the update-only HBM stress (`update_stress`) and the CPU oracle timed on this host
(`cpu_baseline`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # dense MFMA
# HBM-side bytes per launch of the fused weight-gradient kernel at configuration 4 come from a counter run
# (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, scaled by a plain copy kernel of known size); its summary under
# profiles/ carries the figure and the digest of the kernel's sources at the time.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "dual_gemm_bf16_c4_mfma_utilisation_hbm_traffic.txt")
TRAFFIC_SOURCES = ("dw_gemm_bf16.hip", "dw_fused_update.h", "dw_gemm_epi.h", "dw_device_util.h")


def kernel_sources_digest():
    """Digest of the code of the fused weight gradient's sources: comments (the kernels use // only) and white space
    do not count, so rewording a comment does not part the counters from the kernel they were taken on."""
    import hashlib
    import re
    h = hashlib.sha256()
    for f in TRAFFIC_SOURCES:
        text = open(os.path.join(ROOT, "paper_2409_09242_amd", "csrc", f)).read()
        code = [re.sub(r"\s+", " ", re.sub(r"//.*", "", line)).strip() for line in text.splitlines()]
        h.update("\n".join(c for c in code if c).encode())
    return h.hexdigest()[:16]


def measured_traffic():
    """Bytes per launch read from the counter summary, or None when there is none or the kernel's sources have
    changed since the counters were taken (lines `traffic_bytes_per_launch: X` and `kernel_sources_digest: D`)."""
    import re
    try:
        text = open(TRAFFIC_SUMMARY).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, flags=re.M)
    d = re.search(r"^kernel_sources_digest:\s*([0-9a-f]+)", text, flags=re.M)
    if not m or not d or d.group(1) != kernel_sources_digest():
        return None
    return float(m.group(1))


def class_flops(w):
    """Multiply-add work (flop) per all-worker step for each GEMM class."""
    return {c: v * w.k for c, v in w.gemm_flops_by_class().items()}


def fused_layers(w, fuse):
    """Layers whose weight-gradient kernel applies the update itself when fuse_update = 1 (the library's rule:
    W made of whole tiles that fill the chip, averaging block <= 32, Hessian power 1, no convolutional front end)."""
    if not fuse or w.dims is None or w.conv or w.avg_block > 32 or w.hpow != 1.0:
        return []
    tile_n, min_tiles = 128, 512                                   # 128 x 128 tiles in both types
    out, off = [], 0
    for l in range(1, len(w.dims)):
        n_out, n_in = w.dims[l], w.dims[l - 1]
        if (n_out % 128 == 0 and n_in % tile_n == 0 and off % 32 == 0 and n_out * n_in < 2 ** 31
                and (n_out // 128) * (n_in // tile_n) * w.k >= min_tiles):
            out.append(l)
        off += n_out * n_in + n_out
    return out


def r_only_products(w):
    """(forward layers, data-gradient layers) whose products leave out the plain part in the Hutchinson probes after the
    first of a step (the library's rules).  bf16: the products on the global->LDS kernel (whole 256-column tiles that fill
    the chip, contraction a multiple of 128).  fp32: the hidden layers' products whose contraction is not cut into slices
    (at least 256 output tiles over all workers, or a contraction shorter than 128)."""
    if w.dims is None or w.conv:
        return [], []
    d, L = w.dims, len(w.dims) - 1
    if not w.bf16:
        def uncut(rows, n, kk):
            tiles = -(-rows // 128) if n <= 32 else -(-n // 128) if rows <= 32 else -(-rows // 64) * -(-n // 64)
            split = 1024 // (tiles * w.k) if tiles * w.k < 256 else 1
            return min(split, kk // 64, 64) <= 1
        fwd = [l for l in range(1, L) if uncut(w.batch, d[l], d[l - 1])]
        dgrad = [l for l in range(2, L) if uncut(w.batch, d[l - 1], d[l])]
        return fwd, dgrad
    rows = (w.batch + 127) // 128
    off, woff = 0, {}
    for l in range(1, L + 1):
        woff[l] = off
        off += d[l] * d[l - 1] + d[l]
    fwd = [l for l in range(1, L) if w.batch >= 128 and d[l] % 256 == 0 and d[l - 1] % 128 == 0
           and rows * (d[l] // 256) * w.k >= 256 and woff[l] % 128 == 0]
    dgrad = [l for l in range(2, L) if w.batch >= 128 and d[l - 1] % 256 == 0 and d[l] % 128 == 0
             and rows * (d[l - 1] // 256) * w.k >= 256 and woff[l] % 128 == 0]
    return fwd, dgrad


def class_bytes(w, P, k, fused=(), part=1.0, samples=1):
    """Algorithmic HBM bytes per step for the HBM-bound classes.  The update reads g, Hz, theta, m, v and writes
    theta, m, v (32 B per parameter and worker, +2 B for the bf16 weight copy); the pull reads and writes theta
    (8 B per parameter and communicating worker, +2 B bf16 copy; `part` = mean fraction of workers that communicate) and
    the centre (8 B per parameter).  A fused weight-gradient
    launch reads theta, m, v, writes theta, m, v and the bf16 copy (26 B per parameter and worker, + 1 bit of z),
    reads the centre (4 B) on the steps before a round, and reads its four bf16 operands once (d_l, Rd_l, a_{l-1},
    Ra_{l-1}).  With n > 1 Hutchinson probes the fused launches of the first n - 1 probes only keep the running sum
    of z*Hz (first: 4 B written, later: 4 B read and 4 B written per parameter, + 1 bit of z) and the last one
    reads the sum on top of the above (+4 B).  Two probes in bf16 take one launch per layer for both: the state once,
    a second bit of z, six operands instead of four."""
    d = w.dims
    p_fused = sum(d[l] * d[l - 1] for l in fused)
    upd = (32.0 + (2.0 if w.bf16 else 0.0)) * (P - p_fused) * k
    pull = (8.0 + (2.0 if w.bf16 else 0.0)) * P * k * part + 8.0 * P
    out = {"update": upd, "pull": pull}
    if fused:
        es = 2.0 if w.bf16 else 4.0
        operands = sum(2.0 * es * w.batch * (d[l] + d[l - 1]) for l in fused)
        # the centre (4 B) is read only on the steps after which a round is due: one step in tau
        out["gemm_wgrad"] = ((24.125 + (2.0 if w.bf16 else 0.0) + 4.0 / w.tau) * p_fused + operands) * k
        if samples == 2 and w.bf16:
            out["gemm_wgrad"] += (0.125 * p_fused + 0.5 * operands) * k
        elif samples > 1:
            out["gemm_wgrad"] += ((4.125 + 8.125 * (samples - 2) + 4.0) * p_fused + (samples - 1) * operands) * k
    return out


def run_mlp(w, steps, warmup, n_pool, fuse, sequential=False, samples=1, resident=None, repeats=5, zero_data=False):
    import torch
    from paper_2409_09242_amd import binding as B
    from paper_2409_09242_amd import workloads as W

    theta0 = W.init_theta_workload(w)
    x, y = W.minibatch_pool(w, n_pool, bf16_round=W.to_bf16_f32 if w.bf16 else None)
    if zero_data:
        # diagnostic: the same launches on all-zero parameters and inputs, i.e. with the least switching activity
        # in the multipliers and on the data paths; against the run on the workload's own data it shows how much of
        # a kernel's time is set by the clock the power limit leaves it rather than by its instruction schedule
        theta0 = np.zeros_like(theta0)
        x = np.zeros_like(x)
    xd = torch.from_numpy(x).cuda()
    if w.bf16:
        xd = xd.to(torch.bfloat16)
    yd = torch.from_numpy(y).cuda()
    h = B.Handle(B.config_from_workload(w, fuse_update=1 if (fuse and not w.conv) else 0, n_samples=samples), theta0)
    sched = W.participation_schedule(w, ((repeats + 1) * steps + warmup) // w.tau + 2)
    state = {"round": 0, "step": 0}
    mode = B.DW_DYNAMIC | (B.DW_SEQUENTIAL if sequential else 0)

    if resident is not None:
        # the step's input comes from a data set resident in HBM: n points shaped like the workload's inputs, split
        # among the workers with overlap ratio `resident` (Section V-A), every step's minibatch drawn on the device
        n_points = 60000
        gen = torch.Generator(device="cuda"); gen.manual_seed(w.seed)
        data = torch.randn((n_points, w.dims[0]), device="cuda", generator=gen)
        t1 = torch.randn((w.dims[0], 32), device="cuda", generator=gen) / w.dims[0] ** 0.5
        t2 = torch.randn((32, w.dims[-1]), device="cuda", generator=gen) / 32 ** 0.5
        labels = torch.argmax(torch.relu(data @ t1) @ t2, dim=1).to(torch.int32)
        if w.bf16:
            data = data.to(torch.bfloat16)
        index = B.overlap_partition(n_points, int(resident * n_points), w.k, w.seed + 1)
        xb, yb = torch.empty_like(xd[0]), torch.empty_like(yd[0])

    def one_step():
        b = state["step"] % n_pool
        if resident is not None:
            h.draw_batch(data, labels, index, w.seed + 2, xb, yb)
            h.worker_step(xb, yb)
        else:
            h.worker_step(xd[b], yd[b])
        if h.elastic_sync(mode, tau=w.tau, participate=sched[state["round"]]):
            state["round"] += 1
        state["step"] += 1

    for _ in range(warmup):
        one_step()
    # the timed region (exactly `steps` steps between two synchronisations), `repeats` times back to back
    regions = []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            one_step()
        torch.cuda.synchronize()
        regions.append(time.perf_counter() - t0)
    elapsed = float(np.median(regions))

    # second pass over the same number of steps with every launch bracketed by HIP events
    h.profile(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        one_step()
    prof = h.profile_read()
    elapsed_prof = time.perf_counter() - t1
    h.profile(False)
    part = float(np.mean([np.mean(r) for r in sched[:max(state["round"], 1)]]))
    return h, elapsed, prof, elapsed_prof, part, regions


def calibration_copy(n=1 << 28, reps=5):
    """A plain copy of known size (n floats read, n floats written per launch, one elementwise kernel each) so
    that hardware counters collected over this run can be scaled: counter per byte = its reading for this
    kernel / (4 n)."""
    import torch
    src = torch.ones(n, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(reps):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()
    del src, dst
    torch.cuda.empty_cache()


def run_update_stress(iters=20, warmup=3, optimizer=0):
    """Configuration 5: flat P = 1e8 per replica, k = 16; one fused AdaHessian update + one dynamic-weighted
    elastic round per iteration.  Returns GB/s figures against the HBM peak.  optimizer 1 / 2: the same with the
    first-order step of the baselines (SGD: 12 B per parameter and worker, momentum: 20 B, where AdaHessian moves 32)."""
    import torch
    from paper_2409_09242_amd import binding as B
    from paper_2409_09242_amd import workloads as W

    w = W.scaled(W.C5, optimizer=optimizer)
    P, k = w.n_params, w.k
    gen = torch.Generator(device="cuda").manual_seed(w.seed)
    theta0 = (torch.rand(P, device="cuda", generator=gen) - 0.5) * 0.02
    g = torch.randn(k, P, device="cuda", generator=gen) * 0.1
    hz = torch.randn(k, P, device="cuda", generator=gen) * 0.1 if optimizer == 0 else None
    h = B.Handle(B.config_from_workload(w), theta0)
    for _ in range(warmup):
        h.update_only(g, hz)
        h.elastic_sync(B.DW_DYNAMIC, tau=1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        h.update_only(g, hz)
        h.elastic_sync(B.DW_DYNAMIC, tau=1)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    h.profile(True)
    for _ in range(iters):
        h.update_only(g, hz)
        h.elastic_sync(B.DW_DYNAMIC, tau=1)
    prof = h.profile_read()
    h.profile(False)
    by = class_bytes(w, P, k)
    if optimizer:
        by["update"] = (12.0 if optimizer == 1 else 20.0) * P * k
    total_bytes = by["update"] + by["pull"] + 4.0 * P          # + the centre read by the update
    upd_ms = prof["update"][1] / max(prof["update"][0], 1)
    pull_ms = prof["pull"][1] / max(prof["pull"][0], 1)
    out = {
        "workload": w.name, "P": P, "k": k, "iters": iters, "worker_step": ("adahessian", "sgd", "momentum")[optimizer],
        "ms_per_iter": 1e3 * el / iters,
        "bytes_per_iter": total_bytes,
        "GB/s": total_bytes / (el / iters) / 1e9,
        "frac_of_hbm_peak": total_bytes / (el / iters) / 1e9 / PEAK_HBM_GBS,
        "update_kernel": {"ms": upd_ms, "GB/s": by["update"] / (upd_ms * 1e-3) / 1e9,
                          "frac": by["update"] / (upd_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "pull_kernel": {"ms": pull_ms, "GB/s": by["pull"] / (pull_ms * 1e-3) / 1e9,
                        "frac": by["pull"] / (pull_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
    }
    del h, g, hz, theta0
    torch.cuda.empty_cache()
    return out


def hbm_probe(n=1 << 30, reps=20):
    """What HBM sustains for plain streaming kernels of several read : write mixes (torch's elementwise kernels on
    4 GiB arrays; none of the library's code runs): context for the HBM-bound kernels' fractions of the 8 TB/s peak."""
    import torch
    x = torch.ones(n, device="cuda"); y = torch.empty_like(x); z = torch.empty_like(x)
    cases = (("fill (0 read : 1 write)", 1, lambda: y.zero_()), ("copy (1 : 1)", 2, lambda: y.copy_(x)),
             ("add, in place (2 : 1)", 3, lambda: torch.add(x, y, out=y)),
             ("addcmul (3 : 1)", 4, lambda: torch.addcmul(x, y, z, out=z)))
    out = {}
    for name, arrays, f in cases:
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            f()
        torch.cuda.synchronize()
        gbs = arrays * 4.0 * n / ((time.perf_counter() - t0) / reps) / 1e9
        out[name] = {"GB/s": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS}
    return out


def cpu_baseline(w, budget_s=15.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import dw_oracle as O
    from paper_2409_09242_amd import workloads as W
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    est_rate = 2.0e10 * max(cores, 1) / 8.0                    # rough fp64 flop/s, only used to size the sample
    per_worker = w.flops_per_worker_step()
    k_s = int(max(1, min(w.k, budget_s * est_rate / per_worker)))
    ws = W.scaled(w, k=k_s)
    if w.conv:
        # the convolutional oracle has no trainer class: gradient + Hessian-vector product + update per worker
        from oracle import dw_cnn as OC
        from paper_2409_09242_amd import binding as B
        spec = OC.CnnSpec(img=tuple(w.img), conv=tuple(w.conv), fc=tuple(w.dims[1:]))
        idx, _ = B.conv_param_index(w.img, w.conv, w.dims[1:])
        theta = W.init_theta_workload(ws).astype(np.float64)[idx]
        x, y = W.minibatch_pool(ws, 1)
        m, v = np.zeros_like(theta), np.zeros_like(theta)
        z = np.where(W.rng_for(w.seed, 29).random(theta.size) < 0.5, -1.0, 1.0)
        t0 = time.perf_counter()
        n = 0
        while True:
            for i in range(k_s):
                _, g, hz, _ = OC.grad_and_hvp(theta, x[0, i], y[0, i], spec, z)
                theta, m, v = O.adahessian_update(theta, m, v, g, hz, z, n + 1, lr=w.lr, beta1=w.beta1, beta2=w.beta2,
                                                  eps=w.eps, hpow=w.hpow,
                                                  average=(lambda D: OC.spatial_average(D, spec)) if w.conv_avg else None)
            n += 1
            if time.perf_counter() - t0 > budget_s * 0.6 or n >= 50:
                break
        el = time.perf_counter() - t0
        return {"value": k_s * n / el, "unit": "worker-steps/s", "cores": int(cores), "kind": "oracle",
                "sample": "%d of %d workers, %d steps of %s (numpy float64, no communication round)" % (k_s, w.k, n, w.name)}
    theta0 = W.init_theta(ws.dims, ws.seed)
    x, y = W.minibatch_pool(ws, 1, bf16_round=W.to_bf16_f32 if w.bf16 else None)
    tr = O.OracleTrainer(O.OracleConfig(dims=ws.dims, k=k_s, lr=ws.lr, beta1=ws.beta1, beta2=ws.beta2, eps=ws.eps,
                                        hpow=ws.hpow, avg_block=ws.avg_block, alpha=ws.alpha, kappa=ws.kappa,
                                        c=ws.c, seed=ws.seed, bf16=ws.bf16), theta0.astype(np.float64))
    t0 = time.perf_counter()
    n = 0
    while True:
        tr.worker_step(x[0], y[0])
        tr.elastic_sync(O.MODE_DYNAMIC, tau=ws.tau)
        n += 1
        if time.perf_counter() - t0 > budget_s * 0.6 or n >= 50:
            break
    el = time.perf_counter() - t0
    return {"value": k_s * n / el, "unit": "worker-steps/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d of %d workers, %d steps of %s (numpy float64)" % (k_s, w.k, n, w.name)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "cnn"])
    ap.add_argument("--samples", type=int, default=1,
                    help="Rademacher probes per step (n of the Hutchinson estimate; the network runs once per probe)")
    ap.add_argument("--sequential", action="store_true",
                    help="communication rounds as a sequence of single exchanges (DW_SEQUENTIAL); same bytes moved")
    ap.add_argument("--no-fuse", action="store_true",
                    help="keep g and Hz in memory and run the streaming update over all parameters (fuse_update = 0)")
    ap.add_argument("--calibrate", action="store_true",
                    help="first run a plain 1 GiB copy kernel five times (reference for scaling rocprofv3 --pmc counters)")
    ap.add_argument("--resident-data", type=float, default=None, metavar="RATIO",
                    help="draw every step's minibatches on the device from a resident synthetic data set of 60000 "
                         "points, partitioned among the workers with this overlap ratio (e.g. 0.125)")
    ap.add_argument("--zero-data", action="store_true",
                    help="diagnostic: all-zero parameters and inputs (the same launches with the least switching "
                         "activity; shows what the power limit costs on the workload's own data)")
    ap.add_argument("--repeats", type=int, default=5,
                    help="how many times the timed region of --steps steps is run; the line reports the median region")
    ap.add_argument("--no-stress", action="store_true", help="skip the update-only HBM stress (configuration 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hbm-probe", action="store_true",
                    help="run only plain streaming kernels (torch fill, copy, add, addcmul on 4 GiB arrays) and print "
                         "the rates HBM sustains for their read : write mixes")
    ap.add_argument("--stress-only", action="store_true",
                    help="run only the update-only HBM stress and print its figures (for profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the simulated workers are batched on a single device and the library "
              "has no multi-GPU path (--gpus %d refused)" % args.gpus, file=sys.stderr)
        return 2
    if args.zero_data:                       # a diagnostic of the step's kernels: nothing else is run beside it
        args.no_stress = args.no_cpu_baseline = True

    import torch
    from paper_2409_09242_amd import build as BLD
    from paper_2409_09242_amd import workloads as W
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        return 3
    BLD.ensure_built()                      # loads what is built; builds only when nothing is
    if args.hbm_probe:
        print(json.dumps({"hbm_probe": hbm_probe()}))
        return 0
    if args.stress_only:
        print(json.dumps({"update_stress": run_update_stress()}))
        return 0
    w = W.WORKLOADS[args.workload]
    n_pool = 4 if w.bf16 else 8
    if args.calibrate:
        calibration_copy()
    h, elapsed, prof, elapsed_prof, part, regions = run_mlp(w, args.steps, args.warmup, n_pool, not args.no_fuse,
                                                           args.sequential, args.samples, args.resident_data, args.repeats,
                                                           args.zero_data)
    dtype = "bf16" if w.bf16 else "f32"
    ms_per_step = 1e3 * elapsed / args.steps
    value = w.k * args.steps / elapsed

    fl = class_flops(w)
    fused = fused_layers(w, not args.no_fuse)
    skipped = 0.0
    if args.samples > 1:
        fl = {c: v * args.samples for c, v in fl.items()}
        # the fused launches of the probes before the last leave out the plain product (2 B d_l d_{l-1} flop per worker)
        skipped = sum(2.0 * w.batch * w.dims[l] * w.dims[l - 1] for l in fused) * w.k * (args.samples - 1)
        if "gemm_wgrad" in fl:
            fl["gemm_wgrad"] -= skipped
        # and so do the large forward and data-gradient products of the probes after the first
        fwd_r, dgrad_r = r_only_products(w)
        for cls, layers in (("gemm_fwd", fwd_r), ("gemm_dgrad", dgrad_r)):
            less = sum(2.0 * w.batch * w.dims[l] * w.dims[l - 1] for l in layers) * w.k * (args.samples - 1)
            if cls in fl:
                fl[cls] -= less
                skipped += less
    by = class_bytes(w, w.P, w.k, fused, part, args.samples)
    per_step = {"update": 1, "pull": 1.0 / w.tau, "gemm_wgrad": 1, "gather": 1}
    by["gather"] = 2.0 * w.k * w.batch * w.dims[0] * (2 if w.bf16 else 4)        # every drawn row read and written once
    kernels = {}
    for name in ("step", "gemm_fwd", "gemm_wgrad", "gemm_dgrad", "head", "update", "weights", "pull", "rademacher", "gather"):
        n, ms = prof[name]
        if n == 0:
            continue
        entry = {"launches": n, "avg_ms": ms / n, "ms_per_step": ms / args.steps}
        if name in fl:
            entry["TFLOP/s"] = fl[name] / (ms / args.steps * 1e-3) / 1e12
        if name in by:
            # bytes of the class per step over its time per step (the pull runs every tau-th step)
            entry["GB/s"] = by[name] * per_step[name] / (ms / args.steps * 1e-3) / 1e9
        kernels[name] = entry
    if "step" in kernels:
        # a small model's whole step in one kernel: plain fp32 FMA loops out of LDS (no matrix cores)
        kernels["step"]["TFLOP/s"] = sum(fl.values()) / (kernels["step"]["ms_per_step"] * 1e-3) / 1e12
    # classes bound by the matrix cores: all GEMMs, except weight gradients that carry the update (HBM-bound then)
    mfma = [c for c in fl if c in kernels and not (c == "gemm_wgrad" and fused)]
    gemm_ms = sum(kernels[c]["ms_per_step"] for c in mfma)
    gemm_fl = sum(fl[c] for c in mfma)
    dominant = max(kernels, key=lambda c: kernels[c]["ms_per_step"])
    if dominant == "step":
        ach = kernels["step"]["TFLOP/s"]
        roof = {"kernel": "tiny_step_kernel (one block per worker, the whole step)", "bound": "alu", "achieved": ach,
                "peak": PEAK_TFLOPS["f32"], "unit": "TFLOP/s", "frac": ach / PEAK_TFLOPS["f32"], "traffic": None,
                "avg_ms": kernels["step"]["avg_ms"],
                "note": "latency-bound: one compute unit per worker, a chain of dependent phases"}
    elif dominant in mfma:
        # one roofline entry for the GEMM family (one kernel template): all its launches of a step together
        ach = gemm_fl / (gemm_ms * 1e-3) / 1e12
        roof = {"kernel": "dual_gemm (%s)" % dtype, "bound": "mfma", "achieved": ach, "peak": PEAK_TFLOPS[dtype],
                "unit": "TFLOP/s", "frac": ach / PEAK_TFLOPS[dtype], "traffic": None,
                "avg_ms_per_step": gemm_ms, "dominant_class": dominant}
    else:
        ach = kernels[dominant]["GB/s"]
        label = ("dual_gemm_%s weight gradient with fused update" % ("bf16" if w.bf16 else "f32")) if dominant == "gemm_wgrad" else dominant
        roof = {"kernel": label, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": None, "avg_ms": kernels[dominant]["avg_ms"],
                "bytes_per_step": by[dominant] * per_step[dominant]}
        if dominant == "gemm_wgrad":
            # per launch, like the counters: the class has one more, tiny launch per step (the output layer)
            n_big = len(fused) * (1 if (args.samples == 2 and w.bf16) else args.samples)
            roof["launches_per_step"] = n_big
            roof["bytes_per_launch"] = by[dominant] / n_big
            roof["avg_ms"] = kernels[dominant]["ms_per_step"] / n_big
            if w.name.startswith("c4") and args.samples <= 1:
                roof["traffic"] = measured_traffic()
    gemm_roof = None
    if gemm_ms > 0:
        ach_g = gemm_fl / (gemm_ms * 1e-3) / 1e12
        gemm_roof = {"kernel": "dual_gemm (%s): %s, all launches of a step" % (dtype, " + ".join(mfma)),
                     "bound": "mfma", "achieved": ach_g, "peak": PEAK_TFLOPS[dtype], "unit": "TFLOP/s",
                     "frac": ach_g / PEAK_TFLOPS[dtype], "ms_per_step": gemm_ms}
    del h
    torch.cuda.empty_cache()

    out = {
        "metric": "AdaHessian worker-steps/s (incl. Hv)", "value": value, "unit": "worker-steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "timed_regions": len(regions), "ms_per_step_min": 1e3 * min(regions) / args.steps,
        "ms_per_step_max": 1e3 * max(regions) / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype,
        "data": "zeros (diagnostic run, not the workload)" if args.zero_data else "synthetic",
        "config": {"workload": w.name, "k": w.k, "dims": list(w.dims), "batch": w.batch, "tau": w.tau,
                   **({"img": list(w.img), "conv": list(w.conv), "conv_avg": w.conv_avg} if w.conv else {}),
                   "stale": w.stale, "sync": "dynamic, sequential" if args.sequential else "dynamic",
                   "fuse_update": int(bool(fused)), "hutchinson_probes": args.samples,
                   "input": "pool of minibatches" if args.resident_data is None else
                            "drawn on the device from 60000 resident points, overlap %g" % args.resident_data},
        "flop_per_step": w.flops_per_worker_step() * w.k * args.samples - skipped,
        "step_TFLOP/s": (w.flops_per_worker_step() * w.k * args.samples - skipped) / (ms_per_step * 1e-3) / 1e12,
        "ms_per_step_profiled": 1e3 * elapsed_prof / args.steps,
        "roofline": roof,
        "roofline_gemm": gemm_roof,
        "kernels": kernels,
    }
    if not args.no_stress:
        out["update_stress"] = run_update_stress()
        # the first-order worker steps of the baselines (elastic averaging SGD, with and without momentum) on the same vectors
        out["update_stress_baselines"] = [run_update_stress(10, 2, opt) for opt in (1, 2)]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
