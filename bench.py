#!/usr/bin/env python3
"""Benchmark of the tunable-radix non-uniform all-to-all on one MI355X.

A "step" is one whole tuna_alltoallv call (validation, initial rotation, every digit phase:
metadata exchange, scan, pack, exchange, unpack) over one synthetic problem whose send and
receive buffers are already resident in HBM.  Default workload: the P = 4096 flat configuration
(block sizes normal(1 KiB, 256 B), ~16 GiB payload), radix sweep {2, 8, 64, 4096}.

Prints ONE JSON line: `value` is the effective Alltoallv rate (payload bytes / time per call) of
the best radix; `per_radix` has every radix; `roofline` is the dominant copy kernel's achieved
HBM rate (algorithmic bytes = 2 x payload bytes it moves, read + write) against 8 TB/s, timed
with HIP events on the call's stream; `cpu_baseline` is the plain CPU oracle timed on a bounded
sample of the same problem on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch (read + write), averaged over the launches of the default sweep
# (P = 4096, radices 2, 8, 64, 4096: 19 launches of each copy kernel per step set), from two
# `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE), each scaled by what the same counter
# reads for tuna::k_plain_copy moving 4 GiB (factors 2.0000 and 0.9997).  The algorithmic figure
# for the same launches is 2 x payload = 22.55e9 bytes; see profiles/k_copy_config4_P4096.md.
# First entry: T in exact size (the default); second: T in slots of M bytes (--exact-t 0).
MEASURED_TRAFFIC_CONFIG4 = {
    True: {"pack": 22816.4 * 2**20, "exchange": 22307.3 * 2**20, "unpack": 22496.0 * 2**20, "fused": 23689.2 * 2**20},
    False: {"pack": 22847.3 * 2**20, "exchange": 22307.3 * 2**20, "unpack": 22486.3 * 2**20, "fused": 23695.8 * 2**20},
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload configuration 1..5")
    ap.add_argument("--ranks", type=int, default=0, help="override P (reduced-size runs)")
    ap.add_argument("--radices", type=str, default="", help="comma-separated radix sweep")
    ap.add_argument("--element-bytes", type=int, default=8,
                    help="element size of --uniform-max-bytes (8 = the paper's FP64; 16 makes every count and "
                         "displacement a multiple of the 16-byte chunk)")
    ap.add_argument("--uniform-max-bytes", type=int, default=0,
                    help="replace the configuration's counts by 8 * U{0..S/8} bytes (the paper's uniform [0, S] "
                         "micro-benchmark with FP64 elements); use with --ranks and --radices")
    ap.add_argument("--fused", type=int, default=0, help="1: fused single-kernel rounds")
    ap.add_argument("--exact-t", type=int, default=2,
                    help="main sweep, TUNA_OPT_DENSE_T: 2 = the library's default (T in exact size unless the paper's slots "
                         "would be 90 %% full), 1 = exact size, 0 = the paper's B slots of M bytes")
    ap.add_argument("--block-count", type=int, default=0,
                    help="TUNA_OPT_BLOCK_COUNT: rounds per batch of launches (0: all rounds of a phase at once)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fused-table", action="store_true", help="skip the second sweep with fused rounds")
    ap.add_argument("--secondary", action="store_true",
                    help="also sweep the P=1024 hierarchical workload (configuration 3) into also_measured; off by "
                         "default so that every launch of a copy kernel in the run belongs to the timed workload")
    ap.add_argument("--no-secondary", action="store_true", help="accepted for older command lines; the default now")
    ap.add_argument("--no-persistent-table", action="store_true", help="skip the tuna_alltoallv_init / tuna_start sweep")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--traffic-json", type=str, default="",
                    help="optional JSON file {kernel: bytes per launch} from rocprofv3 --pmc runs")
    return ap.parse_args()


def sweep_of(cfg, P):
    import workloads as wl
    c = wl.CONFIGS[cfg]
    if c.global_radices:   # separate local / global radices
        return [("hier", c.ranks_per_node, c.local_radix, rg) for rg in c.global_radices]
    return [("single", c.ranks_per_node, min(r, P), min(r, P)) for r in c.radices]


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all P virtual ranks live in one HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2411_02581_amd as tuna
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    tuna.load()
    dev = "cuda:0"
    cfg = wl.CONFIGS[args.config]
    P = args.ranks or cfg.P
    t0 = time.time()
    if args.uniform_max_bytes:
        counts = wl.counts_uniform_elements(P, cfg.seed, args.uniform_max_bytes // args.element_bytes, args.element_bytes)
    else:
        counts = wl.make_counts(args.config, P)
    lay = wl.make_layout(counts)
    Btot = lay.payload_bytes
    print("[bench] config %d: P=%d payload %.3f GiB, inputs built in %.1f s" %
          (args.config, P, Btot / 2**30, time.time() - t0), file=sys.stderr, flush=True)

    send = wl.payload_position_hash_torch(cfg.seed, lay.send_bytes, dev)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device=dev)
    d_sc = torch.from_numpy(lay.sendcounts).to(dev)
    d_sd = torch.from_numpy(lay.sdispls).to(dev)
    d_rc = torch.from_numpy(lay.recvcounts).to(dev)
    d_rd = torch.from_numpy(lay.rdispls).to(dev)
    torch.cuda.synchronize()

    if args.block_count:
        tuna.tuna_set_option(tuna.TUNA_OPT_BLOCK_COUNT, args.block_count)
    sweep = sweep_of(args.config, P)
    if args.radices:
        rs = [int(x) for x in args.radices.split(",")]
        if cfg.global_radices:
            sweep = [("hier", cfg.ranks_per_node, cfg.local_radix, r) for r in rs]
        else:
            sweep = [("single", cfg.ranks_per_node, min(r, P), min(r, P)) for r in rs]
    rpn = cfg.ranks_per_node if P % max(cfg.ranks_per_node, 1) == 0 else 0

    def call(kind, rl, rg):
        if kind == "hier":
            rc = tuna.tuna_alltoallv_hier(send, d_sc, d_sd, recv, d_rc, d_rd, P, rpn, rl, rg)
        else:
            rc = tuna.tuna_alltoallv(send, d_sc, d_sd, recv, d_rc, d_rd, P, rl, rpn)
        if rc != 0:
            raise RuntimeError("tuna_alltoallv failed: " + tuna.tuna_strerror(rc))

    # ---- practical ceiling: a plain one-chunk-per-thread copy of up to 4 GiB ----------------------
    nb = min(4 << 30, lay.send_bytes // 16 * 16, lay.recv_bytes // 16 * 16)
    copy_ceiling = None
    if nb >= (1 << 20):
        for _ in range(2):
            tuna.tuna_plain_copy(send, recv, nb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            tuna.tuna_plain_copy(send, recv, nb)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        copy_ceiling = {"GBs": 2 * nb / (ms * 1e-3) / 1e9, "bytes_copied": nb, "ms": ms}
        print("[bench] plain copy ceiling: %.0f GB/s (read + write)" % copy_ceiling["GBs"], file=sys.stderr, flush=True)

    def run_sweep(fused, exact_t=2):
        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 1 if fused else 0)
        tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, int(exact_t))
        per_radix = []
        for kind, _, rl, rg in sweep:
            label = "r_l=%d,r_g=%d" % (rl, rg) if kind == "hier" else "r=%d" % rl
            tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 0)
            for _ in range(args.warmup):
                call(kind, rl, rg)
            torch.cuda.synchronize()
            # ---- timed region: exactly K steps between two synchronisations ----------------------
            step_ms = []
            t_start = time.perf_counter()
            for _ in range(args.steps):
                t1 = time.perf_counter()
                call(kind, rl, rg)
                torch.cuda.synchronize()
                step_ms.append((time.perf_counter() - t1) * 1e3)
            torch.cuda.synchronize()
            total_ms = (time.perf_counter() - t_start) * 1e3
            ms_per_step = total_ms / args.steps
            # ---- the same K steps with HIP events around every kernel (roofline figures) ----------
            tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 1)
            kern = {"pack": [0.0, 0, 0], "exchange": [0.0, 0, 0], "unpack": [0.0, 0, 0]}   # ms, launches, payload bytes
            meta_ms = prep_ms = 0.0
            prof_total = 0.0
            for _ in range(args.steps):
                call(kind, rl, rg)
                st = tuna.tuna_get_stats()
                prof_total += st.ms_total
                prep_ms += st.ms_prepare + st.ms_self
                for x in range(st.n_phases):
                    ph = st.phase[x]
                    meta_ms += ph.ms_metadata
                    for name, ms in (("pack", ph.ms_pack), ("exchange", ph.ms_exchange), ("unpack", ph.ms_unpack)):
                        kern[name][0] += ms
                        kern[name][1] += 1
                        kern[name][2] += ph.payload_bytes
            tuna.tuna_set_option(tuna.TUNA_OPT_PROFILE, 0)
            st = tuna.tuna_get_stats()
            hop_bytes = sum(st.phase[x].payload_bytes for x in range(st.n_phases))
            if st.fused:        # one kernel per phase; its time is reported in the pack column
                kern = {"fused": kern["pack"]}
            kernels = {}
            for name, (ms, n, pbytes) in kern.items():
                if n and ms > 0:
                    kernels[name] = {"avg_ms": ms / n, "launches_per_step": n // args.steps,
                                     "alg_bytes_per_launch": 2 * pbytes / n,
                                     "achieved_GBs": 2 * pbytes / (ms * 1e-3) / 1e9}
            per_radix.append({
                "radix": label, "ms_per_step": ms_per_step, "median_ms": statistics.median(step_ms),
                "stdev_ms": statistics.pstdev(step_ms), "effective_GBs": Btot / (ms_per_step * 1e-3) / 1e9,
                "phases": st.n_phases, "rounds": st.K_local + st.K_global, "hop_bytes": hop_bytes,
                "temp_bytes": st.temp_bytes, "workspace_bytes": st.workspace_bytes, "exact_size_t": st.dense_t,
                "profiled_ms_per_step": prof_total / args.steps, "metadata_ms_per_step": meta_ms / args.steps,
                "prepare_ms_per_step": prep_ms / args.steps, "kernels": kernels, "granularity": st.granularity})
            print("[bench] %s: %.3f ms/step, %.1f GB/s effective; " % (label, ms_per_step, per_radix[-1]["effective_GBs"]) +
                  ", ".join("%s %.0f GB/s" % (k, v["achieved_GBs"]) for k, v in kernels.items()) +
              (" [fused rounds]" if fused else ""),
                  file=sys.stderr, flush=True)

        tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 0)
        tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2)
        return per_radix

    def run_persistent(fused, exact_t=2):
        """tuna_alltoallv_init once per radix, then K timed tuna_start calls (no validation, no
        metadata kernels, no host synchronisation), eagerly and as one captured HIP graph.
        exact_t: T stored in exact size (one arena per phase) instead of B slots of M bytes."""
        rows = []
        for kind, _, rl, rg in sweep:
            label = "r_l=%d,r_g=%d" % (rl, rg) if kind == "hier" else "r=%d" % rl
            tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 1 if fused else 0)
            tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, int(exact_t))
            rc, plan = tuna.tuna_alltoallv_init(send, d_sc, d_sd, recv, d_rc, d_rd, P, rpn, rl, rg)
            tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 0)
            tuna.tuna_set_option(tuna.TUNA_OPT_DENSE_T, 2)
            if rc != 0:
                raise RuntimeError("tuna_alltoallv_init failed: " + tuna.tuna_strerror(rc))
            try:
                for _ in range(args.warmup):
                    tuna.tuna_start(plan)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(args.steps):
                    tuna.tuna_start(plan)
                torch.cuda.synchronize()
                ms_start = (time.perf_counter() - t1) * 1e3 / args.steps
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    tuna.tuna_start(plan)
                graph.replay()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(args.steps):
                    graph.replay()
                torch.cuda.synchronize()
                ms_graph = (time.perf_counter() - t1) * 1e3 / args.steps
                del graph
                st = tuna.tuna_get_stats()
                rows.append({"radix": label, "ms_per_start": ms_start, "ms_per_graph_replay": ms_graph,
                             "effective_GBs": Btot / (min(ms_start, ms_graph) * 1e-3) / 1e9,
                             "plan_bytes": st.workspace_bytes, "temp_bytes": st.temp_bytes})
                print("[bench] %s persistent%s%s: %.3f ms/start, %.3f ms/graph replay, %.1f GB/s effective, T %.2f GiB" %
                      (label, " fused" if fused else "", "" if st.dense_t else " slots of M", ms_start, ms_graph,
                       rows[-1]["effective_GBs"], st.temp_bytes / 2 ** 30),
                      file=sys.stderr, flush=True)
            finally:
                tuna.tuna_plan_free(plan)
        return rows

    per_radix = run_sweep(bool(args.fused), args.exact_t)
    # the fused rounds (one kernel per phase, 2 x payload instead of 6 x) as a second table, and both
    # with T in the paper's B slots of M bytes instead of exact size
    fused_table = slots_table = fused_slots_table = None
    if not args.fused and args.exact_t and not args.no_fused_table:
        fused_table = run_sweep(True, args.exact_t)
        slots_table = run_sweep(False, 0)
        fused_slots_table = run_sweep(True, 0)
    persistent = None
    if not args.no_persistent_table:
        persistent = {"note": "tuna_alltoallv_init once, then tuna_start per step: payload kernels only",
                      "staged": run_persistent(bool(args.fused), args.exact_t)}
        if not args.fused and args.exact_t and not args.no_fused_table:
            persistent["fused"] = run_persistent(True, args.exact_t)
            persistent["staged_slots_of_M"] = run_persistent(False, exact_t=0)
            persistent["fused_slots_of_M"] = run_persistent(True, exact_t=0)
    best = max(per_radix, key=lambda r: r["effective_GBs"])
    # Roofline of the dominant kernel: the copy kernel with the largest total time over ALL launches
    # of the timed sweep (every radix), so that its average launch duration is the one a
    # `rocprofv3 --kernel-trace --stats` run of this same command reports for that kernel.
    roofline = None
    tot = {}
    for r in per_radix:
        for name, v in r["kernels"].items():
            t = tot.setdefault(name, [0.0, 0, 0.0])
            n = v["launches_per_step"] * args.steps
            t[0] += v["avg_ms"] * n
            t[1] += n
            t[2] += v["alg_bytes_per_launch"] * n
    if tot:
        gran = per_radix[0]["granularity"]
        dom = max(tot.items(), key=lambda kv: kv[1][0])
        name, (ms, n, alg) = dom
        exact_used = bool(per_radix[0]["exact_size_t"])
        et = "true" if exact_used else "false"
        kname = {"pack": "tuna::k_copy<0, %d, %s>" % (gran, et), "exchange": "tuna::k_copy<1, 16, false>",
                 "unpack": "tuna::k_copy<2, %d, %s>" % (min(gran, 16), et), "fused": "tuna::k_copy<3, %d, %s>" % (gran, et)}[name]
        default_run = (args.config == 4 and P == 4096 and not args.radices)
        traffic = MEASURED_TRAFFIC_CONFIG4[exact_used].get(name) if default_run else None
        achieved = alg / (ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": kname, "stage": name, "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                    "avg_launch_ms": ms / n, "launches": n, "alg_bytes_per_launch": alg / n,
                    "frac_of_plain_copy": (achieved / copy_ceiling["GBs"]) if copy_ceiling else None,
                    "all_stages_GBs": {k: v[2] / (v[0] * 1e-3) / 1e9 for k, v in tot.items()}}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = time_oracle(lay, send, args.cpu_seconds)
        # context, not a target: the GPU call at its best radix against the oracle's plain transpose
        cpu_baseline["gpu_over_cpu"] = {"one_core": best["effective_GBs"] / cpu_baseline["value"],
                                        "all_cores": best["effective_GBs"] / cpu_baseline["all_cores"]["value"]}

    also = None
    if args.secondary and not args.no_secondary:
        also = {"config 3: " + wl.CONFIGS[3].description: quick_sweep(tuna, 3, args.steps, args.warmup)}

    out = {
        "metric": "effective Alltoallv GB/s and % of HBM peak vs radix, at P=1024/4096",
        "metric_note": "value = payload bytes / time per tuna_alltoallv call (three-stage phases) at the best radix of "
                       "the P=4096 workload; per_radix has every radix, roofline the copy kernels' share of the HBM "
                       "peak, also_measured (with --secondary) the P=1024 hierarchical workload",
        "value": best["effective_GBs"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": best["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": ("uniform [0, %d] bytes in %d-byte elements, P=%d flat" % (args.uniform_max_bytes, args.element_bytes, P))
                               if args.uniform_max_bytes else "config %d: %s" % (args.config, cfg.description), "P": P,
                   "payload_bytes": Btot, "best_radix": best["radix"], "fused": bool(args.fused),
                   "exact_size_t": bool(per_radix[0]["exact_size_t"]), "t_layout_option": args.exact_t, "block_count": args.block_count,
                   "ranks_per_node": rpn},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "copy_ceiling": copy_ceiling, "per_radix": per_radix, "persistent": persistent,
        "also_measured": also,
        "fused_rounds": None if fused_table is None else {
            "note": "same workload with TUNA_OPT_FUSED: one kernel per digit phase moves S/T to R/T directly",
            "best_effective_GBs": max(r["effective_GBs"] for r in fused_table), "per_radix": fused_table},
        "slots_of_M": None if slots_table is None else {
            "note": "same workload with TUNA_OPT_DENSE_T = 0: T as the paper's B slots of M bytes per rank instead of exact size",
            "per_radix": slots_table, "fused_per_radix": fused_slots_table},
    }
    print(json.dumps(out))


def quick_sweep(tuna, cfg_id, steps, warmup):
    """Wall-clock sweep of another configuration: immediate calls with three-stage phases and with
    fused rounds, and starts of a persistent plan with fused rounds."""
    import torch

    import workloads as wl
    cfg = wl.CONFIGS[cfg_id]
    lay = wl.make_layout(wl.make_counts(cfg_id))
    dev = "cuda:0"
    send = wl.payload_position_hash_torch(cfg.seed, lay.send_bytes, dev)
    recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device=dev)
    d = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
    rows = []
    for kind, rpn, rl, rg in sweep_of(cfg_id, cfg.P):
        row = {"radix": "r_l=%d,r_g=%d" % (rl, rg) if kind == "hier" else "r=%d" % rl}
        for mode, fused in (("staged", 0), ("fused", 1)):
            tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, fused)
            try:
                def call():
                    if kind == "hier":
                        rc = tuna.tuna_alltoallv_hier(send, d[0], d[1], recv, d[2], d[3], cfg.P, rpn, rl, rg)
                    else:
                        rc = tuna.tuna_alltoallv(send, d[0], d[1], recv, d[2], d[3], cfg.P, rl, rpn)
                    if rc != 0:
                        raise RuntimeError(tuna.tuna_strerror(rc))
                for _ in range(warmup):
                    call()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                for _ in range(steps):
                    call()
                torch.cuda.synchronize()
                ms = (time.perf_counter() - t1) * 1e3 / steps
                row[mode + "_ms"] = ms
                row[mode + "_GBs"] = lay.payload_bytes / (ms * 1e-3) / 1e9
                if fused:
                    rc, plan = tuna.tuna_alltoallv_init(send, d[0], d[1], recv, d[2], d[3], cfg.P, rpn, rl, rg)
                    if rc != 0:
                        raise RuntimeError(tuna.tuna_strerror(rc))
                    try:
                        for _ in range(warmup):
                            tuna.tuna_start(plan)
                        torch.cuda.synchronize()
                        t1 = time.perf_counter()
                        for _ in range(steps):
                            tuna.tuna_start(plan)
                        torch.cuda.synchronize()
                        ms = (time.perf_counter() - t1) * 1e3 / steps
                    finally:
                        tuna.tuna_plan_free(plan)
                    row["persistent_fused_ms"] = ms
                    row["persistent_fused_GBs"] = lay.payload_bytes / (ms * 1e-3) / 1e9
            finally:
                tuna.tuna_set_option(tuna.TUNA_OPT_FUSED, 0)
        rows.append(row)
        print("[bench] config %d %s: staged %.3f ms (%.0f GB/s), fused %.3f ms, persistent fused %.3f ms" %
              (cfg_id, row["radix"], row["staged_ms"], row["staged_GBs"], row["fused_ms"], row["persistent_fused_ms"]),
              file=sys.stderr, flush=True)
    return {"P": cfg.P, "payload_bytes": lay.payload_bytes, "per_radix": rows}


def time_oracle(lay, send_dev, target_seconds):
    """The CPU oracle (plain transpose, one thread) on a bounded sample: the receive side of the
    first n receiver ranks of the same problem, n grown until the run takes about target_seconds."""
    import numpy as np

    import oracle
    t0 = time.time()
    send_host = send_dev.cpu().numpy()
    print("[bench] send buffer to host in %.1f s" % (time.time() - t0), file=sys.stderr, flush=True)
    P = lay.P
    recv_host = np.empty(lay.recv_bytes, dtype=np.uint8)
    recv_host.fill(0)                                        # every page touched before timing
    n = max(1, min(P, P // 64))
    best = None
    spent = 0.0
    while True:
        sel = np.arange(n, dtype=np.int32)
        nbytes = int(lay.recvcounts[:n].astype(np.int64).sum())
        t1 = time.perf_counter()
        rc = oracle.alltoallv_receivers(send_host, lay.sendcounts, lay.sdispls, recv_host, lay.recvcounts,
                                        lay.rdispls, sel)
        dt = time.perf_counter() - t1
        assert rc == 0
        spent += dt
        best = (nbytes, dt, n)
        if n >= P or spent >= target_seconds or dt >= target_seconds / 2:
            break
        scale = (target_seconds / 2) / max(dt, 1e-6)
        n = int(min(P, max(n + 1, n * min(scale, 16))))
    nbytes, dt, n = best
    # the whole workload fits the time budget: repeat it so that about target_seconds of CPU work is timed
    reps = 1
    if n >= P and spent < target_seconds:
        reps = max(1, min(20, int((target_seconds - spent) / max(dt, 1e-6))))
        t1 = time.perf_counter()
        for _ in range(reps):
            oracle.alltoallv_receivers(send_host, lay.sendcounts, lay.sdispls, recv_host, lay.recvcounts,
                                       lay.rdispls, sel)
        dt = (time.perf_counter() - t1) / reps
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    # context only: the same loops split over receiver ranks on all usable host cores
    import threading
    nthr = max(1, min(cores, n))
    parts = np.array_split(np.arange(n, dtype=np.int32), nthr)

    def work(sel):
        oracle.alltoallv_receivers(send_host, lay.sendcounts, lay.sdispls, recv_host, lay.recvcounts, lay.rdispls, sel)
    threads = [threading.Thread(target=work, args=(sel,)) for sel in parts if sel.size]
    t1 = time.perf_counter()
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    dt_par = time.perf_counter() - t1
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle", "cpu_model": model,
            "sample": "receive side of the first %d of %d ranks (%.3f GiB of payload), one thread, %.2f s per pass, "
                      "mean of %d passes; host has %d usable cores" % (n, P, nbytes / 2**30, dt, reps, cores),
            "all_cores": {"value": nbytes / dt_par / 1e9, "unit": "GB/s", "threads": len(threads),
                          "note": "the same oracle called from one thread per slice of receiver ranks"}}


if __name__ == "__main__":
    main()
