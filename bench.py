#!/usr/bin/env python3
"""Benchmark of the tunable-radix non-uniform all-to-all on one MI355X.

A "step" is one whole immediate call (validation, initial rotation, the ranks' own blocks, every
digit phase: metadata exchange, scans, the payload kernels) over one synthetic problem whose send
and receive buffers are already resident in HBM.  Default workload: the P = 4096 flat configuration
(block sizes normal(1 KiB, 256 B), ~16 GiB payload), radix sweep {2, 8, 64, 4096}, with the library's
default options (the mode and the layout of T left to the library).

Prints ONE JSON line:
  value         effective Alltoallv rate (payload bytes / time per call) of the best radix, defaults
  per_radix     every radix of that sweep, with the payload kernels' event-timed rates
  three_stage   the same sweep with pack -> exchange -> unpack as three kernels (the paper's three steps;
                the >= 60 % of HBM peak target is stated for these kernels)
  persistent    tuna_alltoallv_init once, then tuna_start per step
  roofline      the dominant payload kernel of the timed sweep: algorithmic bytes (2 x the payload bytes
                it moves: read + write) / event-timed duration, against 8 TB/s; `traffic` = HBM bytes
                per launch from hardware counters (profiles/traffic_config4_P4096.txt)
  also_measured the P = 1024 hierarchical configuration (the other half of the headline metric) and short
                rows for the staggered schedule, batches of rounds, the FFT count patterns at P = 8192,
                large own blocks and the small-block regime
  cpu_baseline  the plain CPU oracle timed on a bounded sample of the same problem on this machine's cores
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_config4_P4096.txt")
MODES = {"auto": 0, "staged": 1, "fused": 2}
STAGE_OF_MODE = {0: "pack", 1: "exchange", 2: "unpack", 3: "hop"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload configuration 1..5")
    ap.add_argument("--workload", type=str, default="",
                    help="instead of --config: fft_n1 | fft_n2 (the count patterns of the paper's FFT runs) | diagonal "
                         "(64 MiB kept by every rank for itself); use with --ranks")
    ap.add_argument("--ranks", type=int, default=0, help="override P (reduced-size runs)")
    ap.add_argument("--radices", type=str, default="", help="comma-separated radix sweep")
    ap.add_argument("--element-bytes", type=int, default=8,
                    help="element size of --uniform-max-bytes (8 = the paper's FP64; 16 makes every count and "
                         "displacement a multiple of the 16-byte chunk)")
    ap.add_argument("--uniform-max-bytes", type=int, default=0,
                    help="replace the configuration's counts by 8 * U{0..S/8} bytes (the paper's uniform [0, S] "
                         "micro-benchmark with FP64 elements); use with --ranks and --radices")
    ap.add_argument("--mode", choices=sorted(MODES), default="auto",
                    help="main sweep: auto = left to the library (its default), staged = pack / exchange / unpack, "
                         "fused = one kernel per digit phase")
    ap.add_argument("--t-layout", type=int, default=2,
                    help="main sweep, layout of T: 2 = left to the library, 1 = exact size, 0 = the paper's B slots of M bytes")
    ap.add_argument("--staggered", action="store_true", help="main sweep with the staggered inter-node schedule")
    ap.add_argument("--block-count", type=int, default=0,
                    help="rounds per batch of launches (0: all rounds of a phase at once)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-three-stage-table", action="store_true", help="skip the sweep with three-stage phases")
    ap.add_argument("--no-persistent-table", action="store_true", help="skip the tuna_alltoallv_init / tuna_start sweeps")
    ap.add_argument("--no-secondary", action="store_true", help="skip also_measured (configuration 3 and the short rows)")
    ap.add_argument("--slots-table", action="store_true", help="also sweep with T in the paper's slots of M bytes")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--traffic-file", type=str, default=TRAFFIC_FILE,
                    help="text file with the JSON object {kernel name: HBM bytes per launch} of the default run's "
                         "rocprofv3 --pmc passes (lines starting with # are comments)")
    return ap.parse_args()


def load_traffic(path):
    """{kernel name: bytes per launch} and the build id it was measured at, from the tracked summary file."""
    try:
        with open(path) as f:
            text = "".join(line for line in f if not line.lstrip().startswith("#"))
        return json.loads(text)
    except (OSError, ValueError):
        return None


class Resident:
    """One problem resident on the GPU, and timed calls of it."""

    def __init__(self, tuna, counts, seed, ranks_per_node, steps, warmup):
        import torch

        import workloads as wl
        self.tuna, self.torch = tuna, torch
        self.lay = lay = wl.make_layout(counts)
        self.P = lay.P
        self.rpn = ranks_per_node
        self.steps, self.warmup = steps, warmup
        dev = "cuda:0"
        self.send = wl.payload_position_hash_torch(seed, lay.send_bytes, dev)
        self.recv = torch.empty(lay.recv_bytes, dtype=torch.uint8, device=dev)
        self.meta = [torch.from_numpy(a).to(dev) for a in (lay.sendcounts, lay.sdispls, lay.recvcounts, lay.rdispls)]
        self.max_block = int(counts.max()) if counts.size else 0
        # device addresses and the stream resolved once: a timed call is the foreign call, not tensor checks
        sc, sd, rc_, rd = self.meta
        self.ptrs = [t.data_ptr() for t in (self.send, sc, sd, self.recv, rc_, rd)]
        self.stream = torch.cuda.current_stream().cuda_stream
        torch.cuda.synchronize()

    def opts(self, mode=0, t_layout=2, staggered=0, block_count=0, profile=0):
        o = self.tuna.tuna_opts_init()
        o.mode, o.t_layout, o.staggered, o.block_count, o.profile = mode, t_layout, staggered, block_count, profile
        return o

    def call(self, rl, rg, o):
        rc = self.tuna.tuna_alltoallv_ex(None, *self.ptrs, self.P, self.rpn, rl, rg, o, self.stream)
        if rc != 0:
            raise RuntimeError("tuna_alltoallv_ex failed: " + self.tuna.tuna_strerror(rc))

    def time_calls(self, rl, rg, o, label):
        """K timed immediate calls between two synchronisations, then the same K calls with HIP events
        around every kernel (the kernels' rates)."""
        tuna, torch = self.tuna, self.torch
        Btot = self.lay.payload_bytes
        for _ in range(self.warmup):
            self.call(rl, rg, o)
        torch.cuda.synchronize()
        step_ms = []
        t_start = time.perf_counter()
        for _ in range(self.steps):
            t1 = time.perf_counter()
            self.call(rl, rg, o)
            torch.cuda.synchronize()
            step_ms.append((time.perf_counter() - t1) * 1e3)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t_start) * 1e3 / self.steps
        o.profile = 1
        kern = {"pack": [0.0, 0, 0], "exchange": [0.0, 0, 0], "unpack": [0.0, 0, 0], "unpack_last": [0.0, 0, 0]}   # ms, launches, payload bytes
        meta_ms = prep_ms = self_ms = prof_total = 0.0
        for _ in range(self.steps):
            self.call(rl, rg, o)
            st = tuna.tuna_get_stats()
            prof_total += st.ms_total
            prep_ms += st.ms_prepare
            self_ms += st.ms_self
            for x in range(st.n_phases):
                ph = st.phase[x]
                meta_ms += ph.ms_metadata
                # the tiled hop of a schedule's last phase is a kernel variant of its own when the data is word-granular
                last_tiled = bool(st.fused) and x + 1 == st.n_phases and st.granularity < 16
                for name, ms in (("pack", ph.ms_pack), ("exchange", ph.ms_exchange),
                                 ("unpack_last" if last_tiled else "unpack", ph.ms_unpack)):
                    if ms > 0:
                        kern[name][0] += ms
                        kern[name][1] += 1
                        kern[name][2] += ph.payload_bytes
        o.profile = 0
        st = tuna.tuna_get_stats()
        hop_bytes = sum(st.phase[x].payload_bytes for x in range(st.n_phases))
        if st.fused:        # one kernel per phase: the copy engine's hop is reported in the pack column, the
            kern = {"hop": kern["pack"], "tiled_hop": kern["unpack"],     # destination-tiled hop in the unpack column
                    "tiled_hop_last": kern["unpack_last"]}
        else:
            kern.pop("unpack_last")
        kernels = {}
        for name, (ms, n, pbytes) in kern.items():
            if n and ms > 0:
                kernels[name] = {"avg_ms": ms / n, "launches_per_step": n // self.steps,
                                 "alg_bytes_per_launch": 2 * pbytes / n,
                                 "achieved_GBs": 2 * pbytes / (ms * 1e-3) / 1e9}
        row = {"radix": label, "ms_per_step": ms_per_step, "median_ms": statistics.median(step_ms),
               "stdev_ms": statistics.pstdev(step_ms), "effective_GBs": Btot / (ms_per_step * 1e-3) / 1e9,
               "phases": st.n_phases, "rounds": st.K_local + st.K_global, "hop_bytes": hop_bytes,
               "temp_bytes": st.temp_bytes, "workspace_bytes": st.workspace_bytes, "exact_size_t": st.dense_t,
               "one_kernel_phases": st.fused, "profiled_ms_per_step": prof_total / self.steps,
               "metadata_ms_per_step": meta_ms / self.steps, "prepare_ms_per_step": prep_ms / self.steps,
               "own_blocks_ms_per_step": self_ms / self.steps, "kernels": kernels, "granularity": st.granularity,
               "max_block_bytes": int(st.max_block_bytes)}
        print("[bench] %s: %.3f ms/step, %.1f GB/s effective; " % (label, ms_per_step, row["effective_GBs"]) +
              ", ".join("%s %.0f GB/s" % (k, v["achieved_GBs"]) for k, v in kernels.items()) +
              (" [one-kernel phases]" if st.fused else " [three stages]"), file=sys.stderr, flush=True)
        return row

    def sweep(self, radices, **opt):
        return [self.time_calls(rl, rg, self.opts(**opt), label) for label, rl, rg in radices]

    def time_plan(self, rl, rg, o, label):
        """tuna_alltoallv_init once, then K timed tuna_start calls (payload kernels only: no validation,
        no metadata kernels, no host synchronisation), eagerly and as one captured HIP graph."""
        tuna, torch = self.tuna, self.torch
        sc, sd, rc_, rd = self.meta
        rc, plan = tuna.tuna_alltoallv_init_ex(None, self.send, sc, sd, self.recv, rc_, rd, self.P, self.rpn, rl, rg, o)
        if rc != 0:
            raise RuntimeError("tuna_alltoallv_init_ex failed: " + tuna.tuna_strerror(rc))
        try:
            for _ in range(self.warmup):
                tuna.tuna_start(plan)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(self.steps):
                tuna.tuna_start(plan)
            torch.cuda.synchronize()
            ms_start = (time.perf_counter() - t1) * 1e3 / self.steps
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                tuna.tuna_start(plan)
            graph.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(self.steps):
                graph.replay()
            torch.cuda.synchronize()
            ms_graph = (time.perf_counter() - t1) * 1e3 / self.steps
            del graph
            st = tuna.tuna_get_stats()
            row = {"radix": label, "ms_per_start": ms_start, "ms_per_graph_replay": ms_graph,
                   "effective_GBs": self.lay.payload_bytes / (min(ms_start, ms_graph) * 1e-3) / 1e9,
                   "plan_bytes": st.workspace_bytes, "temp_bytes": st.temp_bytes, "one_kernel_phases": st.fused,
                   "exact_size_t": st.dense_t}
            print("[bench] %s persistent%s: %.3f ms/start, %.3f ms/graph replay, %.1f GB/s effective, T %.2f GiB" %
                  (label, " one-kernel" if st.fused else " three stages", ms_start, ms_graph, row["effective_GBs"],
                   st.temp_bytes / 2 ** 30), file=sys.stderr, flush=True)
            return row
        finally:
            tuna.tuna_plan_free(plan)

    def close(self):
        del self.send, self.recv, self.meta
        self.tuna.tuna_release()
        self.torch.cuda.empty_cache()


def radices_of(cfg, P, override=""):
    """[(label, local radix, global radix)] of a configuration's sweep."""
    if override:
        rs = [int(x) for x in override.split(",")]
    elif cfg.global_radices:
        rs = list(cfg.global_radices)
    else:
        rs = list(cfg.radices)
    if cfg.global_radices:
        return [("r_l=%d,r_g=%d" % (cfg.local_radix, r), cfg.local_radix, r) for r in rs]
    return [("r=%d" % min(r, P), min(r, P), min(r, P)) for r in rs]


def kernel_name(stage, gran, exact, max_block_bytes=None):
    et = "true" if exact else "false"
    if stage == "hop" and max_block_bytes is not None and 0 < max_block_bytes <= 64:
        return "tuna::k_hop_small<%d>" % (4 if gran >= 4 else 1)      # one thread per block when all blocks fit into 64 bytes
    return {"pack": "tuna::k_copy<0, %d, %s>" % (gran, et), "exchange": "tuna::k_copy<1, 16, false>",
            "unpack": "tuna::k_copy<2, %d, %s>" % (min(gran, 16), et), "hop": "tuna::k_copy<3, %d, %s>" % (gran, et),
            "tiled_hop": "tuna::k_copy_tiled<%d, 4>" % (16 if gran >= 16 else 4),
            "tiled_hop_last": "tuna::k_copy_tiled<4, 8>"}[stage]


def roofline_of(rows, steps, traffic, copy_ceiling):
    """The payload kernel with the largest total time over ALL launches of the timed sweep (every radix),
    so that its average launch duration is the one `rocprofv3 --kernel-trace --stats` of the same command
    reports for that kernel."""
    tot = {}
    for r in rows:
        for name, v in r["kernels"].items():
            t = tot.setdefault(name, [0.0, 0, 0.0])
            n = v["launches_per_step"] * steps
            t[0] += v["avg_ms"] * n
            t[1] += n
            t[2] += v["alg_bytes_per_launch"] * n
    if not tot:
        return None
    name, (ms, n, alg) = max(tot.items(), key=lambda kv: kv[1][0])
    kname = kernel_name(name, rows[0]["granularity"], bool(rows[0]["exact_size_t"]), rows[0].get("max_block_bytes"))
    achieved = alg / (ms * 1e-3) / 1e9
    tr = traffic.get("bytes_per_launch", {}).get(kname) if traffic else None
    return {"bound": "hbm", "kernel": kname, "stage": name, "achieved": achieved, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": tr,
            "traffic_source": None if tr is None else {"file": "profiles/traffic_config4_P4096.txt",
                                                        "library_build_id": traffic.get("library_build_id")},
            "avg_launch_ms": ms / n, "launches": n, "alg_bytes_per_launch": alg / n,
            "frac_of_plain_copy": (achieved / copy_ceiling["GBs"]) if copy_ceiling else None,
            "all_stages_GBs": {k: v[2] / (v[0] * 1e-3) / 1e9 for k, v in tot.items()}}


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
    cfg = wl.CONFIGS[args.config]
    P = args.ranks or cfg.P
    t0 = time.time()
    if args.workload == "fft_n1":
        counts, wname = wl.counts_fft_n1(P), "FFT count pattern N1 (Section \"Fast Fourier transform\"), P=%d flat" % P
    elif args.workload == "fft_n2":
        counts, wname = wl.counts_fft_n2(P), "FFT count pattern N2 (Section \"Fast Fourier transform\"), P=%d flat" % P
    elif args.workload == "diagonal":
        counts, wname = diagonal_counts(P), "64 MiB kept by every rank for itself, small blocks elsewhere, P=%d flat" % P
    elif args.uniform_max_bytes:
        counts = wl.counts_uniform_elements(P, cfg.seed, args.uniform_max_bytes // args.element_bytes, args.element_bytes)
        wname = "uniform [0, %d] bytes in %d-byte elements, P=%d flat" % (args.uniform_max_bytes, args.element_bytes, P)
    else:
        counts, wname = wl.make_counts(args.config, P), "config %d: %s" % (args.config, cfg.description)
    named = bool(args.workload)
    rpn = 0 if named or args.uniform_max_bytes else (cfg.ranks_per_node if P % max(cfg.ranks_per_node, 1) == 0 else 0)
    res = Resident(tuna, counts, cfg.seed, rpn, args.steps, args.warmup)
    Btot = res.lay.payload_bytes
    print("[bench] %s: P=%d payload %.3f GiB, inputs built in %.1f s, library build %s" %
          (wname, P, Btot / 2**30, time.time() - t0, tuna.tuna_build_id()), file=sys.stderr, flush=True)
    if named or args.uniform_max_bytes:
        rs = [int(x) for x in args.radices.split(",")] if args.radices else [2, P]
        sweep = [("r=%d" % min(r, P), min(r, P), min(r, P)) for r in rs]
    else:
        sweep = radices_of(cfg, P, args.radices)

    # ---- practical ceiling: a plain one-chunk-per-thread copy of up to 4 GiB ----------------------
    nb = min(4 << 30, res.lay.send_bytes // 16 * 16, res.lay.recv_bytes // 16 * 16)
    copy_ceiling = None
    if nb >= (1 << 20):
        for _ in range(2):
            tuna.tuna_plain_copy(res.send, res.recv, nb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            tuna.tuna_plain_copy(res.send, res.recv, nb)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        copy_ceiling = {"GBs": 2 * nb / (ms * 1e-3) / 1e9, "bytes_copied": nb, "ms": ms}
        print("[bench] plain copy ceiling: %.0f GB/s (read + write)" % copy_ceiling["GBs"], file=sys.stderr, flush=True)

    main_opts = dict(mode=MODES[args.mode], t_layout=args.t_layout, staggered=int(args.staggered), block_count=args.block_count)
    per_radix = res.sweep(sweep, **main_opts)
    main_is_staged = not per_radix[0]["one_kernel_phases"]
    three_stage = slots = None
    if not args.no_three_stage_table and not main_is_staged:
        three_stage = res.sweep(sweep, **dict(main_opts, mode=MODES["staged"]))
    if args.slots_table:
        slots = {"note": "T as the paper's B slots of M bytes per rank instead of exact size",
                 "per_radix": res.sweep(sweep, **dict(main_opts, t_layout=0))}
        if three_stage is not None:
            slots["three_stage_per_radix"] = res.sweep(sweep, **dict(main_opts, mode=MODES["staged"], t_layout=0))
    persistent = None
    if not args.no_persistent_table:
        persistent = {"note": "tuna_alltoallv_init once, then tuna_start per step: payload kernels only",
                      "default": [res.time_plan(rl, rg, res.opts(**main_opts), label) for label, rl, rg in sweep]}
        if three_stage is not None:
            persistent["three_stage"] = [res.time_plan(rl, rg, res.opts(**dict(main_opts, mode=MODES["staged"])), label)
                                         for label, rl, rg in sweep]
    best = max(per_radix, key=lambda r: r["effective_GBs"])
    default_run = (args.config == 4 and P == 4096 and not args.radices and not named and not args.uniform_max_bytes
                   and args.mode == "auto" and args.t_layout == 2 and not args.staggered and not args.block_count)
    traffic = load_traffic(args.traffic_file) if default_run else None
    roofline = roofline_of(per_radix, args.steps, traffic, copy_ceiling)
    three_stage_roofline = roofline_of(three_stage, args.steps, traffic, copy_ceiling) if three_stage else None

    # the selector's view of the same problem (built-in constants: nothing is calibrated inside the benchmark)
    rc, ch = tuna.tuna_select(P, rpn, Btot, res.max_block, per_radix[0]["granularity"])
    selector = None if rc != 0 else {"local_radix": ch.local_radix, "global_radix": ch.global_radix,
                                     "mode": "one-kernel phases" if ch.mode == 2 else "three stages",
                                     "t_layout": "exact size" if ch.t_layout == 1 else "slots of M",
                                     "predicted_ms": ch.predicted_ms, "calibrated": bool(ch.calibrated)}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = time_oracle(res.lay, res.send, args.cpu_seconds)
        # context, not a target: the GPU call at its best radix against the oracle's plain transpose
        cpu_baseline["gpu_over_cpu"] = {"one_core": best["effective_GBs"] / cpu_baseline["value"],
                                        "all_cores": best["effective_GBs"] / cpu_baseline["all_cores"]["value"]}
    res.close()

    also = None
    if not args.no_secondary and default_run:
        also = secondary(tuna, wl, np, args, copy_ceiling)

    out = {
        "metric": "effective Alltoallv GB/s and % of HBM peak vs radix, at P=1024/4096",
        "metric_note": "value = payload bytes / time per immediate call with the library's default options at the best radix "
                       "of the P=4096 workload; per_radix has every radix, three_stage the same sweep with pack / exchange / "
                       "unpack as three kernels, roofline the dominant payload kernel's share of the HBM peak, also_measured "
                       "the P=1024 hierarchical workload and short rows for the other schedules",
        "value": best["effective_GBs"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": best["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": wname, "P": P, "payload_bytes": Btot, "best_radix": best["radix"], "mode": args.mode,
                   "one_kernel_phases": bool(best["one_kernel_phases"]), "exact_size_t": bool(best["exact_size_t"]),
                   "t_layout_option": args.t_layout, "staggered": bool(args.staggered), "block_count": args.block_count,
                   "ranks_per_node": rpn, "library_build_id": tuna.tuna_build_id()},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "copy_ceiling": copy_ceiling, "per_radix": per_radix,
        "three_stage": None if three_stage is None else {
            "note": "same workload, pack -> exchange -> unpack as three kernels per digit phase (TUNA_MODE_STAGED)",
            "best_effective_GBs": max(r["effective_GBs"] for r in three_stage), "roofline": three_stage_roofline,
            "per_radix": three_stage},
        "slots_of_M": slots, "persistent": persistent, "selector": selector, "also_measured": also,
    }
    print(json.dumps(out))


def diagonal_counts(P):
    import numpy as np

    import workloads as wl
    counts = wl.counts_uniform_bytes(P, 64, 2000)
    rng = np.random.default_rng(64)
    for p in range(P):
        counts[p, p] = (64 << 20) + 4 * int(rng.integers(-25000, 25000))
    return (counts // 4 * 4).astype(np.int32)


def secondary(tuna, wl, np, args, copy_ceiling):
    """The P = 1024 hierarchical configuration with its own roofline entry, and short rows (few steps) for
    the schedules and workloads the main sweep does not touch."""
    steps, warmup = args.steps, args.warmup
    out = {}
    cfg = wl.CONFIGS[3]
    res = Resident(tuna, wl.make_counts(3), cfg.seed, cfg.ranks_per_node, steps, warmup)
    sweep = radices_of(cfg, cfg.P) + [("r_l=16,r_g=64", 16, 64)]
    rows = res.sweep(sweep)
    staged = res.sweep(sweep, mode=MODES["staged"])
    plans = [res.time_plan(rl, rg, res.opts(), label) for label, rl, rg in sweep]
    best = max(rows, key=lambda r: r["effective_GBs"])
    out["config3"] = {"workload": "config 3: " + cfg.description, "P": cfg.P, "payload_bytes": res.lay.payload_bytes,
                      "value": best["effective_GBs"], "unit": "GB/s", "best_radix": best["radix"], "ms_per_step": best["ms_per_step"],
                      "roofline": roofline_of(rows, steps, None, copy_ceiling), "per_radix": rows,
                      "three_stage": {"roofline": roofline_of(staged, steps, None, copy_ceiling), "per_radix": staged},
                      "persistent": plans}
    # staggered inter-node schedule and batches of rounds on the same problem (Algorithm "Staggered TuNA_l^g";
    # block_count of Algorithm "Coalesced TuNA_l^g")
    short = Resident.__new__(Resident)
    short.__dict__.update(res.__dict__)
    short.steps, short.warmup = max(3, steps // 4), 2
    out["config3"]["staggered"] = short.sweep([("r_l=4 staggered", 4, 64)], staggered=1)
    out["config3"]["block_count"] = [dict(short.time_calls(4, 64, short.opts(block_count=k), "r_l=4,r_g=64 block_count=%d" % k), block_count=k)
                                     for k in (8, 1)]
    res.close()

    def short_rows(name, counts, seed, rpn, sweep, note, **opt):
        r = Resident(tuna, counts, seed, rpn, max(3, steps // 4), 2)
        rows = r.sweep(sweep, **opt)
        plans = [r.time_plan(rl, rg, r.opts(**opt), label) for label, rl, rg in sweep[-1:]]
        out[name] = {"workload": note, "P": r.P, "payload_bytes": r.lay.payload_bytes, "per_radix": rows, "persistent": plans}
        r.close()

    P = 8192
    short_rows("fft_n1", wl.counts_fft_n1(P), 81, 0, [("r=90", 90, 90), ("r=%d" % P, P, P)],
               "FFT count pattern N1 at P=8192: only the ranks below ceil(0.625 P) send, 64 B to each of the first ceil(0.78125 P) ranks")
    short_rows("fft_n2", wl.counts_fft_n2(P), 82, 0, [("r=%d" % P, P, P)],
               "FFT count pattern N2 at P=8192: 512 B per block, 128 B from the last rank")
    short_rows("diagonal", diagonal_counts(64), 83, 0, [("r=64", 64, 64)],
               "64 MiB kept by every rank for itself (P=64), small blocks elsewhere: own_blocks_ms_per_step is the copy of 4 GiB")
    d = out["diagonal"]
    diag_bytes = 64 * (64 << 20)
    d["own_block_copy_GBs"] = [2 * diag_bytes / (r["own_blocks_ms_per_step"] * 1e-3) / 1e9 for r in d["per_radix"]]
    short_rows("small_blocks", wl.counts_uniform_elements(2048, 99, 2, 8), 84, 0, [("r=2", 2, 2), ("r=2048", 2048, 2048)],
               "the paper's uniform [0, 16] bytes at P=2048 (Section \"Performance analysis of TuNA\": small S)")
    short_rows("config1", wl.make_counts(1), wl.CONFIGS[1].seed, 0, [("r=2", 2, 2), ("r=16", 16, 16)],
               "config 1: " + wl.CONFIGS[1].description)
    return out


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
            "all_cores": {"value": nbytes / dt_par / 1e9, "unit": "GB/s", "cores": len(threads), "threads": len(threads),
                          "note": "the same oracle called from one thread per slice of receiver ranks"}}


if __name__ == "__main__":
    main()
