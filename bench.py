#!/usr/bin/env python3
"""Planner benchmark on one MI355X.

A step is one complete plan (prologue, all Jacobi MWU iterations, epilogue) of the largest
benchmark configuration -- 64 modeled nodes x 8 GPUs, 261 632 commodities, 8.3 M candidate
paths, 39.3 M path-link incidences, 1000 iterations -- with topology and traffic resident in
HBM before the timed region.  Prints one JSON line: MWU iterations/s (value), plans/s, the
roofline of the dominant kernel from HIP-event timing, the CPU oracle timed on the host cores
on a bounded sample of the same workload, and (key "also") the throughput of the other
configurations the metric names: the single node, the two-node fabric, the 16-node fabric (one
plan, with its own roofline block, and a batch of 16 plans that share every launch) and the
batch of 4096 single-node plans.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# LDS: 256 compute units x 128 bytes per clock x 2.4 GHz
LDS_PEAK_GBS = 256 * 128 * 2.4
REGIME_NAMES = {1: "resident", 2: "stream", 3: "persistent"}
PHASES = ["argmin", "load_reduce", "update"]


def phase_bytes(lib_topo):
    """Stored bytes each streaming-regime kernel has to move per launch, as the library lays
    the topology out (3.5 or 4 KiB forward records with 8-bit link indices, tile and strip items,
    36-byte reverse octets)."""
    d = {name: lib_topo.phase_bytes(i) for i, name in enumerate(PHASES)}
    d["total"] = lib_topo.bytes_per_iter
    return d


def time_phase(B, torch, h, phase, reps, d_traffic):
    """Average duration of `reps` back-to-back launches of one phase, HIP events on the stream
    the kernels run on (torch's current stream)."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    B.nimble_debug_run_phase(h, phase, 3, d_traffic)
    torch.cuda.synchronize()
    start.record()
    B.nimble_debug_run_phase(h, phase, reps, d_traffic)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e-3 / reps


def time_stream_read(B, torch, nbytes, reps):
    """Read bandwidth (GB/s) of a plain 16-byte-per-lane streaming read of `nbytes`, HIP events
    on torch's current stream around `reps` back-to-back launches."""
    buf = torch.zeros(nbytes // 8, dtype=torch.float64, device="cuda:0")
    sink = torch.zeros(2, dtype=torch.float64, device="cuda:0")
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    B.nimble_debug_stream_read(buf, nbytes, 3, sink)
    torch.cuda.synchronize()
    start.record()
    B.nimble_debug_stream_read(buf, nbytes, reps, sink)
    stop.record()
    torch.cuda.synchronize()
    sec = start.elapsed_time(stop) * 1e-3 / reps
    del buf
    return nbytes / sec / 1e9


def read_traffic(kernel, workload, phase_bytes_now):
    """HBM bytes per launch of `kernel` measured with rocprofv3 counters, from the committed
    summary profiles/hbm_traffic.txt (lines: workload kernel fetch_bytes write_bytes).  The file
    names the stored bytes per phase of the build it was measured on ("# phase_bytes workload
    argmin load_reduce update"); when the running build lays the topology out differently the
    figure is stale and None is returned with a note."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None, "profiles/hbm_traffic.txt is missing"
    value, measured_on = None, None
    for line in open(path):
        parts = line.split()
        if line.startswith("# phase_bytes") and len(parts) >= 6 and parts[2] == workload:
            measured_on = [int(x) for x in parts[3:6]]
        elif len(parts) >= 4 and not line.startswith("#") and parts[0] == workload and \
                parts[1] == kernel:
            value = float(parts[2]) + float(parts[3])
    now = [int(phase_bytes_now[name]) for name in PHASES]
    if measured_on is None:
        return None, "profiles/hbm_traffic.txt does not say which layout it was measured on"
    if measured_on != now:
        return None, (f"profiles/hbm_traffic.txt was measured on a layout of {measured_on} stored "
                      f"bytes per phase, this build has {now}")
    return value, None


def run_config(B, W, torch, cfg, regime, steps, warmup, iters_override=0, batch_size=4096,
               copy_calib=0, plans=0):
    """plans > 0: a batch of that many plans of a single-plan configuration (the configuration's
    own traffic first, then the same recipe with other seeds)."""
    dev = "cuda:0"
    t_gen = time.perf_counter()
    w = W.make_config(cfg, batch=batch_size if cfg == 2 else None)
    topo = w.topo
    if iters_override > 0:
        w.iters = iters_override
    if plans > 0:
        rows = [w.traffic]
        for b in range(1, plans):
            rng = np.random.default_rng(3_000_000 + 1000 * cfg + b)
            rows.append(rng.permutation(w.traffic))      # the same bytes between other pairs
        w.traffic = np.stack(rows)
        w.batch = plans
    t_gen = time.perf_counter() - t_gen
    t_create = time.perf_counter()
    h = B.nimble_topo_create(*topo.csr(), flags=B.NIMBLE_LAYOUT_BATCH if plans > 0 else 0)
    t_create = time.perf_counter() - t_create
    B.nimble_topo_set_regime(h, regime)
    B.nimble_topo_reserve(h, w.iters)       # the choice log, sized outside the timed solves
    batch = max(w.batch, 1)
    if plans > 0:
        B.nimble_topo_reserve_batch(h, plans, w.iters)   # the plans share every launch
    d_traffic = torch.as_tensor(np.ascontiguousarray(w.traffic).reshape(-1)).to(dev)
    d_splits = torch.empty(batch * topo.n_paths, dtype=torch.float64, device=dev)
    d_lambda = torch.empty(batch, dtype=torch.float64, device=dev)

    def step():
        if w.batch:
            B.nimble_plan_solve_batch(h, batch, d_traffic, w.eps, w.iters, d_splits, d_lambda)
        else:
            B.nimble_plan_solve(h, d_traffic, w.eps, w.iters, d_splits, d_lambda)

    if copy_calib > 0:      # plain device copies of 1 GiB: calibration of the HBM counters
        src = torch.empty(1 << 27, dtype=torch.float64, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(copy_calib):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    return dict(w=w, topo=topo, h=h, batch=batch, d_traffic=d_traffic, d_splits=d_splits,
                d_lambda=d_lambda, elapsed=elapsed, event_s=ev0.elapsed_time(ev1) * 1e-3,
                regime=h.regime, t_gen=t_gen, t_create=t_create)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 0..4")
    ap.add_argument("--regime", type=int, default=0,
                    help="0 auto, 1 resident, 2 stream, 3 persistent")
    ap.add_argument("--cpu-iters", type=int, default=-1,
                    help="oracle iterations for the CPU baseline (-1: sized to ~15 s, 0: skip)")
    ap.add_argument("--batch", type=int, default=4096)
    ap.add_argument("--iters", type=int, default=0,
                    help="override the configuration's iteration count (profiling runs only)")
    ap.add_argument("--copy-calib", type=int, default=0,
                    help="also run N plain device copies of 1 GiB (counter calibration)")
    ap.add_argument("--plans", type=int, default=0,
                    help="run a batch of N plans of a single-plan configuration (profiling runs)")
    ap.add_argument("--no-barrier-probe", action="store_true",
                    help="skip the grid-barrier probe (its cooperative launch makes rocprofv3 "
                         "crash when the traced process exits)")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the extra configurations reported under 'also'")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the planner models the whole "
              "fabric on one device); --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    from paper_2604_00317_amd import binding as B
    from paper_2604_00317_amd import workloads as W
    B.load_library(build_if_missing=True)

    r = run_config(B, W, torch, args.config, args.regime, args.steps, args.warmup, args.iters,
                   args.batch, args.copy_calib, plans=args.plans)
    w, topo, h, batch = r["w"], r["topo"], r["h"], r["batch"]
    elapsed, regime = r["elapsed"], r["regime"]
    ms_per_step = elapsed * 1e3 / args.steps
    iters_per_s = w.iters * batch * args.steps / elapsed
    plans_per_s = batch * args.steps / elapsed
    lam = r["d_lambda"].cpu().numpy()
    workload = f"configs[{args.config}] {w.name}" + (f" x{args.plans}" if args.plans else "")

    # ---- roofline of the dominant kernel ------------------------------------------------
    bytes_ = phase_bytes(h)
    kernels = {}
    if regime == B.NIMBLE_REGIME_STREAM:
        for ph, name in enumerate(PHASES):
            if bytes_[name] == 0:        # the length update runs inside the reduce kernel
                continue
            # (a batch: the launches of one plan, the first)
            sec = time_phase(B, torch, h, ph, 200, r["d_traffic"][:topo.n_comm])
            if name == "load_reduce" and bytes_["update"] == 0:
                name = "reduce_update"
            kernels[name] = dict(back_to_back_us=sec * 1e6, bytes=bytes_[PHASES[ph]])
        # Launched one after the other inside a plan the kernels take longer than when one
        # kernel is launched again and again (each starts on what the previous, different,
        # kernel has just written), and rocprofv3's dispatch times tile the plan without gaps.
        # avg_us is therefore the kernel's share of the measured time per iteration, split in
        # proportion to the back-to-back averages: the duration a launch has where it counts.
        per_iter_us = elapsed / args.steps / w.iters * 1e6
        scale = per_iter_us / sum(k["back_to_back_us"] for k in kernels.values())
        for k in kernels.values():
            k["avg_us"] = k["back_to_back_us"] * scale
            k["gbs"] = k["bytes"] / k["avg_us"] / 1e3
            k["back_to_back_gbs"] = k["bytes"] / k["back_to_back_us"] / 1e3
        dom = max(kernels, key=lambda n: kernels[n]["avg_us"])
        traffic, traffic_note = read_traffic(dom, w.name, bytes_)
        whole = bytes_["total"] * w.iters * args.steps / elapsed / 1e9
        roofline = dict(bound="hbm", kernel=dom, achieved=kernels[dom]["gbs"],
                        peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=kernels[dom]["gbs"] / HBM_PEAK_GBS,
                        back_to_back_achieved=kernels[dom]["back_to_back_gbs"],
                        back_to_back_frac=kernels[dom]["back_to_back_gbs"] / HBM_PEAK_GBS,
                        traffic=traffic,
                        whole_iteration_gbs=whole, whole_iteration_frac=whole / HBM_PEAK_GBS,
                        bytes=kernels[dom]["bytes"],
                        note=("stored bytes are re-read every iteration and fit the 256 MB "
                              "Infinity Cache: the rate is cache-resident bandwidth, priced "
                              "against the HBM peak"))
        if traffic_note:
            roofline["traffic_note"] = traffic_note
        # what the path-cost kernel gathers from LDS (one 8-byte price per candidate step): the
        # resource nearest its limit once the forward bytes are compressed
        lds_bytes = h.phase_bytes(3)
        if lds_bytes > 0 and "argmin" in kernels:
            lds_gbs = lds_bytes / kernels["argmin"]["avg_us"] / 1e3
            roofline["lds_gather"] = dict(kernel="argmin", bytes=lds_bytes, achieved=lds_gbs,
                                          peak=LDS_PEAK_GBS, unit="GB/s",
                                          frac=lds_gbs / LDS_PEAK_GBS)
        # the same iteration rate priced at the bytes an uncompressed layout (32-bit indices,
        # one reverse entry per incidence) would have to move: context for the compression
        plain = (8 * topo.nnz + 4 * topo.n_paths + 4 * topo.n_links + 24 * topo.n_comm +
                 48 * topo.n_links)
        # what a plain streaming read reaches on this machine: a buffer far beyond the 256 MB
        # Infinity Cache (HBM), and one of the dominant kernel's own size (re-read every launch,
        # as the kernel's data is, so served by the Infinity Cache)
        hbm_read = time_stream_read(B, torch, 2 << 30, 20)
        own = max(int(kernels[dom]["bytes"]) // 16 * 16, 1 << 20)
        own_read = time_stream_read(B, torch, own, 100)
        roofline["empirical_read"] = dict(
            unit="GB/s", buffer_2GiB=hbm_read, buffer_of_kernel_size=own_read,
            kernel_bytes=own, frac_of_2GiB_read=kernels[dom]["gbs"] / hbm_read,
            frac_of_same_size_read=kernels[dom]["gbs"] / own_read)
        roofline["plain_csr_bytes_per_iter"] = int(plain)
        roofline["plain_csr_equivalent_gbs"] = plain * w.iters * args.steps / elapsed / 1e9
    else:
        # one kernel per step: its duration is the step time measured with HIP events
        sec = r["event_s"] / args.steps
        total = bytes_["total"] * w.iters * batch
        name = REGIME_NAMES.get(regime, "auto")
        roofline = dict(bound="hbm", kernel=name, achieved=total / sec / 1e9, peak=HBM_PEAK_GBS,
                        unit="GB/s", frac=total / sec / 1e9 / HBM_PEAK_GBS,
                        traffic=None)

    # ---- CPU baseline: the oracle on a bounded sample -------------------------------------
    cpu = None
    if args.cpu_iters != 0:
        import oracle
        cores = oracle.max_threads()
        if w.batch:
            n_plans = 64 if args.cpu_iters < 0 else max(1, args.cpu_iters)
            n_plans = min(n_plans, batch)
            t1 = time.perf_counter()
            worst = 0.0
            for b in range(n_plans):
                ref = oracle.solve(*topo.csr(), w.traffic[b], w.eps, w.iters)
                worst = max(worst, abs(lam[b] - ref["lam"]) / max(ref["lam"], 1e-300))
            dt = time.perf_counter() - t1
            cpu = dict(value=w.iters * n_plans / dt, unit="iterations/s", cores=cores,
                       kind="oracle", plans_per_s=n_plans / dt,
                       sample=f"first {n_plans} of {batch} plans, all {w.iters} iterations",
                       max_rel_diff_lambda=worst)
        else:
            n_it = args.cpu_iters
            if n_it < 0:
                oracle.solve(*topo.csr(), w.traffic, w.eps, 1)          # page everything in
                t1 = time.perf_counter()
                oracle.solve(*topo.csr(), w.traffic, w.eps, 4)
                per_it = (time.perf_counter() - t1) / 4
                n_it = int(max(4, min(w.iters, 15.0 / max(per_it, 1e-6))))
            t1 = time.perf_counter()
            ref = oracle.solve(*topo.csr(), w.traffic, w.eps, n_it)
            dt = time.perf_counter() - t1
            # parity of the same shortened run on the GPU
            B.nimble_plan_solve(h, r["d_traffic"], w.eps, n_it, r["d_splits"], r["d_lambda"])
            torch.cuda.synchronize()
            g_s = r["d_splits"].cpu().numpy()
            g_l = float(r["d_lambda"].item())
            cpu = dict(value=n_it / dt, unit="iterations/s", cores=cores, kind="oracle",
                       plans_per_s=1.0 / (dt * w.iters / n_it),
                       sample=f"first {n_it} of {w.iters} iterations, all commodities",
                       max_abs_diff_splits=float(np.abs(g_s - ref["splits"]).max()),
                       max_rel_diff_lambda=abs(g_l - ref["lam"]) / max(ref["lam"], 1e-300))
    setup = {"generate": r["t_gen"], "topo_create": r["t_create"]}

    # ---- post-processing of the plan into byte flows per path (whole chunks) ----------------
    post = None
    if not w.batch and not args.no_also:
        n_it = w.iters
        B.nimble_plan_solve(h, r["d_traffic"], w.eps, n_it, r["d_splits"], r["d_lambda"])
        chi, theta = 1 << 20, float(1 << 20)
        d_flows = torch.empty(topo.n_paths, dtype=torch.float64, device="cuda:0")
        B.nimble_plan_quantize(h, r["d_traffic"], r["d_splits"], n_it, chi, theta, d_flows)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(20):
            B.nimble_plan_quantize(h, r["d_traffic"], r["d_splits"], n_it, chi, theta, d_flows)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t1) / 20
        post = dict(kernel="quantize", us_per_plan=dt * 1e6, chi=chi, small_threshold=theta,
                    bytes=int(16 * topo.n_paths + 12 * topo.n_comm),
                    gbs=(16 * topo.n_paths + 12 * topo.n_comm) / dt / 1e9)
        if args.cpu_iters != 0:
            import oracle
            n_k = min(topo.n_comm, 20000)           # the Python oracle on the first pairs
            cp = topo.comm_path_ptr[:n_k + 1]
            sp = r["d_splits"].cpu().numpy()
            t1 = time.perf_counter()
            ref = oracle.quantize(cp, w.traffic[:n_k], sp[:cp[-1]], n_it, chi, theta)
            dtc = time.perf_counter() - t1
            got = d_flows.cpu().numpy()[:cp[-1]]
            post["cpu_oracle_us_per_plan"] = dtc * 1e6 * topo.n_comm / n_k
            post["cpu_sample"] = f"first {n_k} of {topo.n_comm} pairs, one core, scaled"
            post["max_abs_diff_flows"] = float(np.abs(got - ref).max())
    # ---- adaptive step + early stop on the same workload -------------------------------------
    adaptive = None
    if not w.batch and not args.no_also:
        B.nimble_plan_solve(h, r["d_traffic"], w.eps, w.iters, r["d_splits"], r["d_lambda"])
        torch.cuda.synchronize()
        lam_fixed = float(r["d_lambda"].item())
        check_every = 25
        B.nimble_plan_solve_adaptive(h, r["d_traffic"], w.eps, 4 * w.iters, check_every,
                                     r["d_splits"], r["d_lambda"])          # warm-up
        t1 = time.perf_counter()
        n_done, lb = B.nimble_plan_solve_adaptive(h, r["d_traffic"], w.eps, 4 * w.iters,
                                                  check_every, r["d_splits"], r["d_lambda"])
        dt = time.perf_counter() - t1
        lam_ad = float(r["d_lambda"].item())
        adaptive = dict(iterations=n_done, ms_per_plan=dt * 1e3, iterations_per_s=n_done / dt,
                        us_per_iteration=dt * 1e6 / n_done,
                        check_every=check_every, lambda_=lam_ad, lower_bound=lb,
                        gap=lam_ad / lb if lb > 0 else None, target_gap=(1 + w.eps) ** 2,
                        lambda_fixed_step=lam_fixed, fixed_step_iters=w.iters,
                        fixed_step_ms=ms_per_step,
                        launches_per_iteration=2 if h.adaptive_folds else 3)
    h.close()
    del r

    # ---- the other throughput figures the metric names -------------------------------------
    also = {}
    if not args.no_also and args.config == 4 and args.iters == 0:
        single_c3 = None
        for cfg, steps, plans in ((0, 20, 0), (1, 20, 0), (3, 5, 0), (3, 3, 16), (2, 5, 0)):
            q = run_config(B, W, torch, cfg, 0, steps, 1, 0, args.batch, plans=plans)
            key = f"configs[{cfg}] {q['w'].name}" + (f" x{plans}" if plans else "")
            entry = dict(
                iterations_per_s=q["w"].iters * q["batch"] * steps / q["elapsed"],
                plans_per_s=q["batch"] * steps / q["elapsed"],
                ms_per_step=q["elapsed"] * 1e3 / steps,
                us_per_iteration=q["elapsed"] * 1e6 / steps / q["w"].iters,
                regime=REGIME_NAMES.get(q["regime"], "auto"), batch=q["batch"],
                iters=q["w"].iters)
            also[key] = entry
            if cfg == 3 and not plans:
                # the 16-node fabric, named by the bandwidth target as well: its 5 MB per
                # iteration stay in the caches, two dependent launches per iteration
                single_c3 = entry["plans_per_s"]
                b3 = phase_bytes(q["h"])
                gbs = b3["total"] * q["w"].iters * steps / q["elapsed"] / 1e9
                entry["roofline"] = dict(bound="hbm", bytes_per_iter=b3["total"],
                                         us_per_iter=entry["us_per_iteration"], achieved=gbs,
                                         peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS,
                                         note="cache-resident; bound by two grid-wide "
                                              "dependencies per iteration, not by bandwidth")
                ks = {}
                for ph, name in enumerate(PHASES):
                    if b3[name]:
                        sec = time_phase(B, torch, q["h"], ph, 200, q["d_traffic"])
                        ks["reduce_update" if ph == 1 and not b3["update"] else name] = dict(
                            back_to_back_us=sec * 1e6, bytes=b3[name])
                entry["kernels"] = ks
                # the adaptive step on the same fabric (two launches per iteration where the
                # step is applied inside the next record kernel, else three)
                ws = q["w"]
                for _ in range(2):
                    torch.cuda.synchronize()
                    t1 = time.perf_counter()
                    n_ad, lb_ad = B.nimble_plan_solve_adaptive(
                        q["h"], q["d_traffic"], ws.eps, 4 * ws.iters, 25, q["d_splits"],
                        q["d_lambda"])
                    dt_ad = time.perf_counter() - t1
                entry["adaptive_step"] = dict(iterations=n_ad, ms_per_plan=dt_ad * 1e3,
                                              us_per_iteration=dt_ad * 1e6 / n_ad, check_every=25,
                                              lower_bound=lb_ad,
                                              lambda_=float(q["d_lambda"].item()),
                                              launches_per_iteration=2 if q["h"].adaptive_folds
                                              else 3)
            if cfg == 3 and plans and single_c3:
                entry["speedup_over_one_plan_at_a_time"] = entry["plans_per_s"] / single_c3
            if cfg == 2:
                # the paper's own sequential planner (Algorithm 1) on the same batch: one GPU
                # thread per problem; lambda against the Jacobi MWU plan of the same problems
                phi, chi = 0.5, float(1 << 20)
                nb, P = q["batch"], q["topo"].n_paths
                d_flows = torch.empty(nb * P, dtype=torch.float64, device="cuda:0")
                d_lam1 = torch.empty(nb, dtype=torch.float64, device="cuda:0")
                d_sw = torch.empty(nb, dtype=torch.int32, device="cuda:0")

                def alg1_step():
                    B.nimble_alg1_solve_batch(q["h"], nb, q["d_traffic"], phi, chi, 1 << 20,
                                              d_flows, d_lam1, d_sw)
                alg1_step()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(steps):
                    alg1_step()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t1
                ratio = (d_lam1 / q["d_lambda"]).cpu().numpy()
                entry = dict(plans_per_s=nb * steps / dt, ms_per_step=dt * 1e3 / steps, batch=nb,
                             phi=phi, chi=chi, mean_sweeps=float(d_sw.float().mean().item()),
                             lambda_over_mwu_mean=float(ratio.mean()),
                             lambda_over_mwu_max=float(ratio.max()))
                if args.cpu_iters != 0:
                    import oracle
                    n_cpu = min(nb, 256)
                    t1 = time.perf_counter()
                    worst = 0.0
                    lam1 = d_lam1.cpu().numpy()
                    for b in range(n_cpu):
                        ref = oracle.alg1(*q["topo"].csr(), q["w"].traffic[b], phi, chi)
                        worst = max(worst, abs(lam1[b] - ref["lam"]))
                    dtc = time.perf_counter() - t1
                    entry["cpu_oracle_plans_per_s"] = n_cpu / dtc
                    entry["cpu_sample"] = f"first {n_cpu} of {nb} problems, one core"
                    entry["max_abs_diff_lambda"] = worst
                also[f"configs[{cfg}] {q['w'].name} (Algorithm 1)"] = entry
            q["h"].close()
            del q

    # ---- what a grid-wide barrier costs next to the kernel boundaries the plan uses -----------
    barrier = None
    if not args.no_also and not args.no_barrier_probe:
        work = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
        res = torch.zeros(32, dtype=torch.int32, device="cuda:0")
        barrier = {}
        for kind, name in ((0, "flat_counter"), (1, "flat_counter_with_fences"),
                           (2, "counter_per_xcd")):
            for bpc in (1, 4):
                B.nimble_debug_barrier_probe(kind, bpc, 256, 20, 1 << 16, work, res)
                torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                B.nimble_debug_barrier_probe(kind, bpc, 256, 250, 1 << 16, work, res)
                e1.record()
                torch.cuda.synchronize()
                o = res.cpu().numpy()
                barrier[f"{name}_{bpc}_per_cu_us"] = (
                    e0.elapsed_time(e1) * 1e3 / 500 if o[0] == 0 and o[1] == 0 else None)
        del work, res

    out = {
        "metric": "mwu_iterations_per_s", "value": iters_per_s, "unit": "iterations/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": workload, "commodities": topo.n_comm, "paths": topo.n_paths,
                   "incidences": topo.nnz, "links": topo.n_links, "eps": w.eps, "iters": w.iters,
                   "batch": batch, "regime": REGIME_NAMES.get(regime, "auto")},
        "plans_per_s": plans_per_s,
        "lambda": float(lam[0]),
        "bytes_per_iter": bytes_["total"],
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": cpu,
        "also": also,
        "post_processing": post,
        "adaptive_step": adaptive,
        "grid_barrier": barrier,
        "setup_s": setup,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
