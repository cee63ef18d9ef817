#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: persistent isomorphic all-to-all and
allgather with the message-combining (torus-direct) schedule, one kernel per
round, on synthetic workloads held entirely in HBM.

One step = one iso_start of every collective the workload names (e.g. config 5:
all-to-all, then allgather), enqueued back to back on one stream.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line on stdout;
everything else goes to stderr.

Default run: the headline numbers (`value`, `roofline`, `cpu_baseline`) are taken on
the largest workload, config 5 (8^5 torus, 40 neighbours, 4 KiB blocks, 5.4 GB per
buffer); the other workloads whose blocks are at least 128 bytes (configs 2, 3 and
4) are timed the same way in the same run and reported under `workloads`, each with
its own roofline and CPU baseline; `small_blocks` lists config 4's torus at 16, 32
and 64 bytes with the plain and the staged schedule, and `comparison` (on config 2)
the other algorithms, layouts and interfaces.  `--config N` times one workload only.
`roofline.traffic` is counted by the run itself: after a workload is timed, two child
runs of this program on that workload under `rocprofv3 --pmc` (FETCH_SIZE, then
WRITE_SIZE); `--no-live-traffic` reports the recorded summary under profiles/ instead.
"""
import argparse
import csv
import glob
import json
import os
import shutil
import signal
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak, GB/s
LAST_LEVEL_CACHE_BYTES = 256 << 20
METRIC = "delivered GB/s (p*s*m bytes per collective / time) at 1 GPU; % of HBM peak"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default=None,
                    help="time only this workload (1..5); default: config 5 as the headline, then 2, 3 and 4")
    ap.add_argument("--m", type=int, default=None, help="override the block size in bytes (with --config)")
    ap.add_argument("--layout", choices=("rank", "slot"), default="rank",
                    help="buffers of the timed requests: rank = the paper's [p][s][m] (default), slot = [s][p][m]")
    ap.add_argument("--algorithm", choices=("combined", "bydim", "sx_fused", "sx_rounds", "onehop", "staged"),
                    default="combined", help="algorithm of the timed requests (default: combined, one kernel per round)")
    ap.add_argument("--pad", type=int, default=0,
                    help="all-to-all only: every rank's row padded by this many bytes (irregular interface, equal blocks)")
    ap.add_argument("--mesh", action="store_true", help="the torus taken as a box: no dimension wraps (Section 7)")
    ap.add_argument("--irregular", type=int, default=0, metavar="BASE",
                    help="all-to-all with the stencil block sizes of Section 4: BASE^(d - |C|_1) bytes per neighbour")
    ap.add_argument("--graph", type=int, default=0, choices=(0, 1, 2),
                    help="replay the timed requests as HIP graphs: 1 = chain of kernel nodes, 2 = rounds of one "
                         "dimension as parallel branches")
    ap.add_argument("--seed", type=int, default=2016)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the comparison algorithms and the copy ceiling")
    ap.add_argument("--timed-only", action="store_true",
                    help="only the timed region: no isolated repetitions, no per-round timing (for counter runs)")
    ap.add_argument("--copy-reference", action="store_true",
                    help="with --no-extras: still run the 1 GiB plain copy (calibration of the traffic counters)")
    ap.add_argument("--cpu-seconds", type=float, default=6.0, help="CPU-oracle timing budget per workload")
    ap.add_argument("--no-live-traffic", action="store_true",
                    help="do not count HBM traffic in child runs under rocprofv3; `roofline.traffic` then comes "
                         "from the recorded summary under profiles/ (implied by --timed-only)")
    ap.add_argument("--small-sweep", action="store_true",
                    help="instead of the benchmark: all-to-all on tori of about 500 processes (the paper's own "
                         "regime, Section 4), every algorithm, three block sizes; prints one JSON line")
    ap.add_argument("--setup-times", action="store_true",
                    help="instead of the benchmark: times of the host steps (neighbourhood, schedule, init) for the "
                         "Moore neighbourhoods of the paper's set-up table (Section 4); prints one JSON line")
    return ap.parse_args()


def recorded_traffic(tag):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of
    this same command (the summary whose name carries `tag`) and that file's name, else
    (None, None).  Stands in where the traffic is not counted by the run itself."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", f"*{tag}_hbm_traffic.txt"))):
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return int(line.split("=")[1]), "recorded: profiles/" + os.path.basename(path)
    return None, None


def scaled_counter_average(csv_path, counter):
    """From rocprofv3's counter_collection.csv: the average of `counter` (KiB per dispatch) over the
    library's kernels other than the plain copy, scaled so that the plain copy's own average
    reads 1 GiB = 2^20 KiB (what it moves each way), and that scale; None if either kind of
    dispatch is missing."""
    copy, rounds = [], []
    for row in csv.DictReader(open(csv_path)):
        if row["Counter_Name"] != counter or "iso::" not in row["Kernel_Name"]:
            continue
        (copy if "copy_kernel" in row["Kernel_Name"] else rounds).append(float(row["Counter_Value"]))
    if not copy or not rounds:
        return None
    scale = (1 << 20) / (sum(copy) / len(copy))
    return sum(rounds) / len(rounds) * scale, scale


def counted_kib(command, counter):
    """Runs `command` (this program with --timed-only --copy-reference) under
    `rocprofv3 --pmc <counter>` and returns the counter's average per dispatch of the
    library's kernels of the step, scaled by what it reads for the plain copy of 1 GiB
    in the same run, as (KiB per launch, scale); None if the run fails."""
    out_dir = tempfile.mkdtemp(prefix="iso_pmc_", dir="/tmp")
    env = dict(os.environ, TMPDIR="/tmp")
    full = ["timeout", "-s", "KILL", "150", "rocprofv3", "--pmc", counter, "--output-format", "csv",
            "-d", out_dir, "-o", "x", "--"] + command
    try:
        child = subprocess.Popen(full, cwd="/tmp", env=env, stdout=subprocess.DEVNULL, stderr=subprocess.PIPE,
                                 start_new_session=True)
        try:
            _, err = child.communicate(timeout=170)
        except subprocess.TimeoutExpired:
            os.killpg(child.pid, signal.SIGKILL)         # the group this call started, nothing else
            child.communicate()
            log(f"  live traffic: {counter} run exceeded its time limit")
            return None
        if child.returncode != 0:
            log(f"  live traffic: {counter} run ended with status {child.returncode}: "
                f"{err.decode(errors='replace')[-300:]}")
            return None
        files = glob.glob(os.path.join(out_dir, "**", "*counter_collection.csv"), recursive=True)
        if not files:
            return None
        return scaled_counter_average(files[0], counter)
    except OSError as e:                                 # no profiler on this machine
        log(f"  live traffic: {e}")
        return None
    finally:
        shutil.rmtree(out_dir, ignore_errors=True)


def live_traffic(flags):
    """HBM bytes per launch of the step's kernels, counted now: two child runs of this program
    with `flags` under rocprofv3, FETCH_SIZE then WRITE_SIZE (KiB per dispatch, one counter per
    run), each scaled by the same counter's reading for the plain 1 GiB copy.  None if either
    run fails."""
    command = ["python3", os.path.join(ROOT, "bench.py")] + flags + [
        "--steps", "3", "--warmup", "1", "--timed-only", "--no-cpu-baseline", "--no-extras", "--copy-reference"]
    fetch = counted_kib(command, "FETCH_SIZE")
    write = counted_kib(command, "WRITE_SIZE") if fetch else None
    if not fetch or not write:
        return None
    return {"bytes_per_launch": int((fetch[0] + write[0]) * 1024),
            "fetched": int(fetch[0] * 1024), "written": int(write[0] * 1024),
            "copy_scale": [round(fetch[1], 4), round(write[1], 4)]}


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def small_sweep():
    """Section 4's setting carried over: Moore neighbourhoods on tori of about 500 processes,
    block sizes from a few bytes to 2 KiB.  Here every size is bound by the per-launch cost, the
    GPU's counterpart of the message start-up latency, so the time follows the number of launches:
    D for the message-combining schedules, s for the straightforward algorithm."""
    import numpy as np
    import torch
    import iso_inputs as gen
    import paper_1606_07676_amd as iso
    iso.load_library()
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    algs = (("combined", iso.ISO_ALG_COMBINED), ("combined_bydim", iso.ISO_ALG_COMBINED_BYDIM),
            ("combined_staged", iso.ISO_ALG_COMBINED_STAGED), ("onehop", iso.ISO_ALG_ONEHOP), ("sx_rounds", iso.ISO_ALG_SX_ROUNDS), ("sx_fused", iso.ISO_ALG_SX_FUSED))
    cases = (("moore_d2_r1", (30, 16), gen.moore(2, 1)), ("moore_d3_r1", (8, 8, 8), gen.moore(3, 1)),
             ("moore_d4_r1", (6, 5, 4, 4), gen.moore(4, 1)), ("moore_d5_r1", (4,) * 5, gen.moore(5, 1)),
             ("moore_d3_r3", (8, 8, 8), gen.moore(3, 3)), ("shales_d3_r3_r7", (9, 8, 8), gen.shales(3, (3, 7))))
    rows = []
    for name, dims, offs in cases:
        p, s = int(np.prod(dims)), len(offs)
        comm = iso.iso_neighborhood_create(dims, offs)
        for m in (16, 256, 2048):
            send = gen.alltoall_send_torch(1, p, s, m, device=dev)
            recv = torch.empty((p, s, m), dtype=torch.uint8, device=dev)
            row = {"neighbourhood": name, "dims": list(dims), "p": p, "s": s, "m": m}
            for an, alg in algs:
                wsb = iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, alg, m)
                work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                req = iso.iso_neighbor_alltoall_init(send, recv, m, work, comm, alg)
                for graph in (iso.ISO_GRAPH_OFF, iso.ISO_GRAPH_CHAIN):
                    iso.iso_request_set_graph(req, graph)
                    for _ in range(10):
                        iso.iso_start(req, stream)
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for _ in range(200):
                        iso.iso_start(req, stream)
                    e1.record(stream)
                    torch.cuda.synchronize()
                    if graph:
                        row[an]["graph_us"] = round(e0.elapsed_time(e1) / 200 * 1e3, 2)
                    else:
                        row[an] = {"us": round(e0.elapsed_time(e1) / 200 * 1e3, 2),
                                   "launches": iso.iso_request_info(req)["launches"]}
                iso.iso_request_free(req)
            log(row)
            rows.append(row)
    print(json.dumps({"small_sweep": rows}), flush=True)


def setup_times():
    """Section 4's set-up table carried over: full Moore neighbourhoods of radius 1 to 3 in 2 to 5
    dimensions on a torus of 480 processes (30 x 16 there; factored evenly per dimension here).
    Times of the host steps, median of 25 calls each, ms: iso_neighborhood_create (validation,
    residues, round lists), the schedule computation alone (iso_plan_create, all-to-all and
    allgather), and iso_neighbor_alltoall_init on device buffers (schedule, checks of the buffers,
    table built and copied to the device)."""
    import numpy as np
    import torch
    import iso_inputs as gen
    import paper_1606_07676_amd as iso
    iso.load_library()
    dev = "cuda:0"
    torus = {2: (24, 20), 3: (10, 8, 6), 4: (6, 5, 4, 4), 5: (5, 4, 4, 3, 2)}
    m, reps = 8, 25

    def timed(fn, free=None):
        ts = []
        for _ in range(reps):
            t0 = time.perf_counter()
            obj = fn()
            ts.append((time.perf_counter() - t0) * 1e3)
            if free:
                free(obj)
        return round(median(ts), 4)

    rows = []
    for d in (2, 3, 4, 5):
        for r in (1, 2, 3):
            dims, offs = torus[d], np.asarray(gen.moore(d, r), np.int32)
            p, s_n = int(np.prod(dims)), len(offs)
            comm = iso.iso_neighborhood_create(dims, offs)
            send = torch.zeros((p, s_n, m), dtype=torch.uint8, device=dev)
            recv = torch.empty_like(send)
            work = torch.empty(max(iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m), 16),
                               dtype=torch.uint8, device=dev)
            row = {"d": d, "radius": r, "dims": list(dims), "s": s_n,
                   "iso_neighborhood_create_ms": timed(lambda: iso.iso_neighborhood_create(dims, offs)),
                   "schedule_alltoall_ms": timed(lambda: iso.iso_plan_create(comm, iso.ISO_OP_ALLTOALL,
                                                                            iso.ISO_ALG_COMBINED), iso.iso_plan_free),
                   "schedule_allgather_ms": timed(lambda: iso.iso_plan_create(comm, iso.ISO_OP_ALLGATHER,
                                                                             iso.ISO_ALG_COMBINED), iso.iso_plan_free),
                   "iso_neighbor_alltoall_init_ms": timed(lambda: iso.iso_neighbor_alltoall_init(send, recv, m, work, comm),
                                                          iso.iso_request_free)}
            req = iso.iso_neighbor_alltoall_init(send, recv, m, work, comm)
            row["rounds"] = iso.iso_request_info(req)["launches"]
            iso.iso_request_free(req)
            log(row)
            rows.append(row)
    print(json.dumps({"setup_times": rows}), flush=True)


class Bench:
    """One workload on the device: buffers, requests, timing, the CPU-oracle leg."""
    host_threads = 0           # threads the C oracle used on its first (default) call
    arena = None               # the run's one device allocation (see __init__)
    ALIGN = 2 << 20

    @staticmethod
    def arena_need(iso, comm, ops, p, s, m, slot, alg):
        need = 0
        for op in ops:
            a2a = op == iso.ISO_OP_ALLTOALL
            need += ((p * s * m if a2a else p * m) + p * s * m) * (2 if slot else 1) + 4 * Bench.ALIGN
            need += iso.iso_workspace_bytes(comm, op, alg, m) + Bench.ALIGN
        return need

    def __init__(self, args, cfg, m):
        import numpy as np
        import torch
        import iso_inputs as gen
        import paper_1606_07676_amd as iso
        self.np, self.torch, self.gen, self.iso = np, torch, gen, iso
        self.args, self.cfg, self.m = args, cfg, m
        self.dev = "cuda:0"
        self.stream = torch.cuda.current_stream()
        self.p, self.s = cfg.p, cfg.s
        self.slot = args.layout == "slot"
        self.alg = {"combined": iso.ISO_ALG_COMBINED, "bydim": iso.ISO_ALG_COMBINED_BYDIM,
                    "sx_fused": iso.ISO_ALG_SX_FUSED, "sx_rounds": iso.ISO_ALG_SX_ROUNDS,
                    "onehop": iso.ISO_ALG_ONEHOP, "staged": iso.ISO_ALG_COMBINED_STAGED}[args.algorithm]
        self.plain = not (args.mesh or args.irregular or args.pad)      # the CPU leg covers these only
        self.op_name = {iso.ISO_OP_ALLTOALL: "alltoall", iso.ISO_OP_ALLGATHER: "allgather"}
        self.ops = [iso.ISO_OP_ALLTOALL if o == "alltoall" else iso.ISO_OP_ALLGATHER for o in cfg.ops]
        if not self.plain:
            self.ops = [iso.ISO_OP_ALLTOALL]
        self.keep = []

        t0 = time.perf_counter()
        if args.mesh:
            self.comm = iso.iso_neighborhood_create_mesh(cfg.dims, (0,) * cfg.d, cfg.offsets)
        else:
            self.comm = iso.iso_neighborhood_create(cfg.dims, cfg.offsets)
        self.t_create = (time.perf_counter() - t0) * 1e3
        self.cinfo = iso.iso_neighborhood_info(self.comm)

        p, s, dev = self.p, self.s, self.dev
        self.bufs, self.timed = {}, {}
        # One device allocation for the whole run, made before anything else touches device memory;
        # the buffers of the timed requests are carved from it at 2 MiB boundaries.  A single large
        # allocation made first is physically contiguous, separate mid-sized ones made after tens
        # of GB have been allocated and freed need not be, and where the blocks of a round sit in
        # physical memory decides how evenly they load the memory channels (config 3: 0.58 - 0.69 of
        # peak on separate allocations after such churn, 0.67 - 0.70 on one allocation).
        ALIGN = Bench.ALIGN
        if self.plain:
            need = Bench.arena_need(iso, self.comm, self.ops, p, s, m, self.slot, self.alg)
            if Bench.arena is None or Bench.arena.numel() < need + ALIGN:
                Bench.arena = None
                Bench.arena = torch.empty(need + ALIGN, dtype=torch.uint8, device=dev)
            self.arena = Bench.arena
            self.arena_at = (-self.arena.data_ptr()) % ALIGN

        def take(nbytes):
            lo = self.arena_at
            self.arena_at = lo + -(-nbytes // ALIGN) * ALIGN
            assert self.arena_at <= self.arena.numel()
            return self.arena[lo:lo + nbytes]
        self.take = take
        if self.plain:
            for op in self.ops:
                if op == iso.ISO_OP_ALLTOALL:
                    send = gen.alltoall_send_torch(args.seed, p, s, m, cfg.kind, device=dev, out=take(p * s * m).view(p, s, m))
                else:
                    send = take(p * m).view(p, m)
                    send.copy_(gen.allgather_send_torch(args.seed, p, m, cfg.kind, device=dev))
                recv = take(p * s * m).view(p, s, m).fill_(0xEE)
                self.bufs[op] = (send, recv)
            for op in self.ops:               # with --layout slot the same blocks as [s][p][m]
                send, recv = self.bufs[op]
                if self.slot:
                    if op == iso.ISO_OP_ALLTOALL:
                        tsend = take(p * s * m).view(s, p, m)
                        tsend.copy_(send.permute(1, 0, 2))
                    else:
                        tsend = send
                    self.timed[op] = (tsend, take(p * s * m).view(s, p, m).fill_(0xEE))
                else:
                    self.timed[op] = (send, recv)
        self.footprint = 0
        self.reqs, self.t_init = [], []
        for op in self.ops:
            r, t = self.make_request(op, self.alg, timed_buffers=True)
            self.reqs.append(r)
            self.t_init.append(t)
        self.infos = [iso.iso_request_info(r) for r in self.reqs]
        self.delivered = sum(i["delivered_bytes"] for i in self.infos)
        self.moved = sum(i["bytes_read"] + i["bytes_written"] for i in self.infos)
        self.launches = sum(i["launches"] for i in self.infos)
        if args.graph:
            for r in self.reqs:
                iso.iso_request_set_graph(r, args.graph)

    # -- requests ------------------------------------------------------------------
    def make_request(self, op, alg, timed_buffers=False):
        iso, torch, gen, args = self.iso, self.torch, self.gen, self.args
        p, s, m, dev = self.p, self.s, self.m, self.dev
        if not self.plain:                                 # irregular interface: padded rows or stencil sizes
            if args.irregular:
                sizes = gen.stencil_block_sizes(self.cfg.offsets, args.irregular)
                displs, ext = gen.packed_displacements(sizes, 16)
            else:
                sizes, displs, ext = [m] * s, [i * m for i in range(s)], s * m
            ext += args.pad
            wsb = iso.iso_workspace_bytes_v(self.comm, op, alg, sizes)
            work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
            if self.slot:
                pd, at = [], 0
                for sz in sizes:
                    pd.append(at)
                    at += -(-p * sz // 16) * 16
                send = torch.empty(at, dtype=torch.uint8, device=dev).fill_(3)
                recv = torch.empty(at, dtype=torch.uint8, device=dev)
                torch.cuda.synchronize()
                t = time.perf_counter()
                req = iso.iso_neighbor_alltoallv_init_layout(send, sizes, pd, 0, recv, sizes, pd, 0,
                                                             iso.ISO_LAYOUT_SLOT_MAJOR, work, self.comm, alg)
            else:
                send = torch.empty((p, ext), dtype=torch.uint8, device=dev).fill_(3)
                recv = torch.empty((p, ext), dtype=torch.uint8, device=dev)
                torch.cuda.synchronize()
                t = time.perf_counter()
                req = iso.iso_neighbor_alltoallv_init(send, sizes, displs, ext, recv, sizes, displs, ext,
                                                      work, self.comm, alg)
            dt = (time.perf_counter() - t) * 1e3
            self.keep += [send, recv, work]
            self.footprint += send.numel() + recv.numel() + wsb
            return req, dt
        send, recv = self.timed[op] if timed_buffers else self.bufs[op]
        wsb = iso.iso_workspace_bytes(self.comm, op, alg, m)
        if timed_buffers:
            work = self.take(wsb) if wsb else None
        else:
            work = torch.empty(wsb, dtype=torch.uint8, device=dev) if wsb else None
        init = iso.iso_neighbor_alltoall_init_layout if op == iso.ISO_OP_ALLTOALL else \
            iso.iso_neighbor_allgather_init_layout
        layout = iso.ISO_LAYOUT_SLOT_MAJOR if (timed_buffers and self.slot) else iso.ISO_LAYOUT_RANK_MAJOR
        torch.cuda.synchronize()                 # the init call copies its table synchronously: keep the fills out of its time
        t = time.perf_counter()
        req = init(send, recv, m, layout, work, self.comm, alg)
        dt = (time.perf_counter() - t) * 1e3
        if timed_buffers:
            self.footprint += send.numel() + recv.numel() + wsb
        return req, dt

    def time_steps(self, reqs, steps, warmup):
        iso, torch, stream = self.iso, self.torch, self.stream
        for _ in range(warmup):
            for r in reqs:
                iso.iso_start(r, stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            for r in reqs:
                iso.iso_start(r, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)                         # ms for `steps` steps

    # -- the timed region and what is derived from it ---------------------------------
    def run(self):
        iso, torch, args, cfg = self.iso, self.torch, self.args, self.cfg
        K, W, m, p, s = args.steps, args.warmup, self.m, self.p, self.s
        reqs, infos, stream = self.reqs, self.infos, self.stream
        log(f"workload {cfg.name}: dims={cfg.dims} p={p} s={s} m={m} ops={[self.op_name[o] for o in self.ops]} "
            f"algorithm={args.algorithm} layout={args.layout}")
        total_ms = self.time_steps(reqs, K, W)
        ms_per_step = total_ms / K
        value = self.delivered / (ms_per_step * 1e-3) / 1e9
        log(f"  {ms_per_step:.4f} ms/step, delivered {value:.1f} GB/s, moved "
            f"{self.moved / (ms_per_step * 1e-3) / 1e9:.1f} GB/s over {self.launches} launches")

        # the paper's measurement protocol (Section 4): every repetition timed on its own after a
        # synchronisation, outliers outside [Q1 - 3 IQR, Q3 + 3 IQR] dropped, median kept
        reps = 0 if args.timed_only else 100
        rep_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in rep_ev:
            torch.cuda.synchronize()
            a.record(stream)
            for r in reqs:
                iso.iso_start(r, stream)
            b.record(stream)
        torch.cuda.synchronize()
        protocol = None
        if reps:
            rep_ms = sorted(a.elapsed_time(b) for a, b in rep_ev)
            q1, q3 = rep_ms[reps // 4], rep_ms[(3 * reps) // 4]
            kept = [t for t in rep_ms if q1 - 3 * (q3 - q1) <= t <= q3 + 3 * (q3 - q1)]
            protocol = {"repetitions": reps, "kept_after_tukey_3iqr": len(kept), "median_ms": round(median(kept), 5),
                        "min_ms": round(kept[0], 5), "max_ms": round(kept[-1], 5),
                        "delivered_GBs_at_median": round(self.delivered / median(kept) / 1e6, 1)}

        # per-launch durations (HIP events on the launch stream around single launches; these
        # include the event markers themselves and are listed for orientation)
        per_round = []
        ev_steps = max(1, min(K, 30))
        for r, inf in zip(reqs, infos):
            if args.timed_only:
                break
            plan = iso.iso_request_plan(r)
            n = inf["launches"]
            n_rounds = iso.iso_plan_info(plan)["launches"]
            if n != n_rounds:          # a round was split over several launches: no per-round listing
                continue
            ks = [iso.iso_plan_round(plan, q)["n_entries"] for q in range(n)]
            dims_ = [iso.iso_plan_round(plan, q)["dim"] for q in range(n)]
            evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                    for _ in range(n)] for _ in range(ev_steps)]
            torch.cuda.synchronize()
            for st in range(ev_steps):
                for q in range(n):
                    a, b = evs[st][q]
                    a.record(stream)
                    iso.iso_start_range(r, q, 1, stream)
                    b.record(stream)
            torch.cuda.synchronize()
            uniform = not args.irregular
            for q in range(n):
                t_ms = median([evs[st][q][0].elapsed_time(evs[st][q][1]) for st in range(ev_steps)])
                row = {"op": self.op_name[inf["op"]], "round": q, "dim": dims_[q], "k": ks[q],
                       "us": round(t_ms * 1e3, 2)}
                if uniform:
                    row["moved_GBs"] = round(2 * ks[q] * p * m / (t_ms * 1e-3) / 1e9, 1)
                per_round.append(row)

        # Every launch of the step is the same kernel, so its average launch duration over the
        # timed region is region time / launches in the region (gaps between back-to-back
        # launches included).
        alg_bytes_per_launch = self.moved / self.launches
        avg_launch_ms = ms_per_step / self.launches
        achieved = alg_bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
        kernel = ("vector_round_kernel" if args.algorithm.startswith("sx") else
                  "deliver_kernel" if args.algorithm == "staged" and m % 16 == 0 and s * (m // 16) <= 2048 and s <= 128
                  and not (args.irregular or args.mesh or args.pad or self.slot) else
                  "block_round_kernel" if args.irregular else
                  "mesh_shift_round_kernel" if args.mesh else
                  "shift_round_uniform_kernel" if m % 1024 == 0 and (self.slot or m <= 2048) else
                  "shift_round_kernel") + "<16B>"
        tag = self.tag()
        roofline = {
            "kernel": kernel, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": recorded_traffic(tag)[0], "traffic_source": recorded_traffic(tag)[1],
            "algorithmic_bytes_per_launch": int(alg_bytes_per_launch),
            "avg_launch_us": round(avg_launch_ms * 1e3, 2), "launches_per_step": self.launches,
        }
        out = {
            "value": round(value, 2), "unit": "GB/s", "ms_per_step": round(ms_per_step, 5),
            "config": {
                "workload": f"{cfg.name if m == cfg.m else cfg.name.rsplit('_m', 1)[0] + f'_m{m}'}: torus "
                            f"{'x'.join(map(str, cfg.dims))} (p={p}), s={s}, m={m} B, "
                            f"{'+'.join(self.op_name[o] for o in self.ops)} per step, "
                            + ("message-combining schedule, one kernel per round" if args.algorithm == "combined"
                               else f"algorithm {args.algorithm}"),
                "layout": "[s][p][m] (slot-major)" if self.slot else "[p][s][m] (rank-major, the paper's)",
                "algorithm": args.algorithm, "seed": args.seed, "profile_tag": tag,
                "rounds": self.cinfo["rounds"], "delivered_bytes_per_step": self.delivered,
                "moved_bytes_per_step": self.moved,
                "device_footprint_bytes": int(self.footprint),
                "exceeds_last_level_cache": bool(self.footprint > LAST_LEVEL_CACHE_BYTES),
            },
            "verified_against_oracle": None,      # set by the CPU-oracle leg
            "roofline": roofline,
            "isolated_repetitions": protocol,
            "per_round": per_round,
            "setup_ms": {"iso_neighborhood_create": round(self.t_create, 4),
                         **{f"iso_neighbor_{self.op_name[op]}_init": round(t, 4)
                            for op, t in zip(self.ops, self.t_init)}},
        }
        for key, flag in (("mesh", args.mesh), ("irregular_base", args.irregular), ("row_padding", args.pad),
                          ("graph", args.graph)):
            if flag:
                out["config"][key] = flag
        return out

    def flags(self):
        """The command-line flags that time this workload and variant alone."""
        a = self.args
        f = ["--config", str(self.gen.CONFIGS.index(self.cfg) + 1), "--m", str(self.m), "--algorithm", a.algorithm,
             "--layout", a.layout, "--seed", str(a.seed)]
        if a.mesh:
            f.append("--mesh")
        for name, value in (("--irregular", a.irregular), ("--pad", a.pad), ("--graph", a.graph)):
            if value:
                f += [name, str(value)]
        return f

    def tag(self):
        """Names the (workload, variant) in the file names under profiles/."""
        a = self.args
        t = f"c{self.gen.CONFIGS.index(self.cfg) + 1}_m{self.m}"
        if a.algorithm != "combined":
            t += f"_{a.algorithm}"
        if self.slot:
            t += "_slot"
        if a.mesh:
            t += "_mesh"
        if a.irregular:
            t += f"_stencil{a.irregular}"
        if a.pad:
            t += f"_pad{a.pad}"
        return t

    def copy_reference_rate(self):
        """GB/s read + written by the library's plain copy kernel on 1 GiB: the ceiling, and the
        copy of known size that the HBM traffic counters are calibrated on."""
        iso, torch, stream = self.iso, self.torch, self.stream
        nb = 1 << 30
        a = torch.empty(nb, dtype=torch.uint8, device=self.dev)
        b = torch.empty(nb, dtype=torch.uint8, device=self.dev)
        for _ in range(3):
            iso.iso_copy_reference(a, b, nb, stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(20):
            iso.iso_copy_reference(a, b, nb, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        return round(2 * nb * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)

    # -- comparison algorithms (not part of `value`) ------------------------------------
    def comparison(self):
        iso, torch, gen, args, cfg = self.iso, self.torch, self.gen, self.args, self.cfg
        p, s, m, dev, ops, comm = self.p, self.s, self.m, self.dev, self.ops, self.comm
        K = args.steps
        extras = {}
        ksteps = max(5, K // 4)

        def rate(rs, ms, hbm_label=True):
            """`moved_GBs` counts the bytes the algorithm asks for (read + written), which is
            what HBM carries for the message-combining schedules (every block is read once and
            written once per hop).  The s-exchange allgather reads each source block s times,
            mostly from cache, so for it the figure is not HBM traffic and gets no fraction."""
            mv = sum(iso.iso_request_info(r)["bytes_read"] * 2 for r in rs)
            dl = sum(iso.iso_request_info(r)["delivered_bytes"] for r in rs)
            d = {"ms_per_step": round(ms, 5), "delivered_GBs": round(dl / ms / 1e6, 1),
                 "launches": sum(iso.iso_request_info(r)["launches"] for r in rs)}
            if hbm_label:
                d["moved_GBs"] = round(mv / ms / 1e6, 1)
                d["frac_of_peak"] = round(mv / ms / 1e6 / HBM_PEAK_GBS, 4)
            else:
                d["requested_GBs_not_hbm"] = round(mv / ms / 1e6, 1)
            return d

        for name, alg in (("combined_bydim", iso.ISO_ALG_COMBINED_BYDIM), ("sx_fused", iso.ISO_ALG_SX_FUSED),
                          ("sx_rounds", iso.ISO_ALG_SX_ROUNDS), ("onehop", iso.ISO_ALG_ONEHOP)):
            rs = [self.make_request(op, alg)[0] for op in ops]
            ms = self.time_steps(rs, ksteps, 3) / ksteps
            extras[name] = rate(rs, ms, hbm_label=not (name.startswith("sx") and iso.ISO_OP_ALLGATHER in ops))
            for r in rs:
                iso.iso_request_free(r)
        for op, r in zip(ops, self.reqs):
            ms = self.time_steps([r], ksteps, 3) / ksteps
            extras[f"combined_{self.op_name[op]}_only"] = rate([r], ms)
        for form, name in ((iso.ISO_GRAPH_CHAIN, "combined_graph_chain"), (iso.ISO_GRAPH_BRANCHES, "combined_graph_branches")):
            for r in self.reqs:                              # the same requests replayed as HIP graphs
                iso.iso_request_set_graph(r, form)
            ms = self.time_steps(self.reqs, ksteps, 3) / ksteps
            extras[name] = rate(self.reqs, ms)
            extras[name]["launches"] = len(self.reqs)
        for r in self.reqs:
            iso.iso_request_set_graph(r, iso.ISO_GRAPH_OFF)
        extras["copy_1GiB_GBs_read_plus_write"] = self.copy_reference_rate()
        # irregular all-to-all in the shape of the paper's stencil experiment (Section 4): block of
        # neighbour i has base^(d - ||C^i||_1) bytes; same torus, Moore radius 1, base 64
        if cfg.d == 3 and cfg is gen.get_config(2):
            offs = gen.moore(3, 1)
            sizes = gen.stencil_block_sizes(offs, 64)
            icomm = iso.iso_neighborhood_create(cfg.dims, offs)
            # blocks in neighbour order at 16-byte aligned displacements; packed back to back (rows of
            # 25352 bytes); and, same row length as the first, the large blocks side by side at the start of
            # the row with the tiny ones packed behind them (a choice of the caller's displacements)
            for tag, align in (("", 16), ("packed_", 1), ("large_blocks_first_", 16)):
                displs, ext = gen.packed_displacements(sizes, align)
                if tag == "large_blocks_first_":
                    at = 0
                    for i in sorted(range(len(sizes)), key=lambda i: -sizes[i]):
                        displs[i] = at
                        at += -(-sizes[i] // 16) * 16
                isend = torch.empty((p, ext), dtype=torch.uint8, device=dev).fill_(3)
                irecv = torch.empty((p, ext), dtype=torch.uint8, device=dev)
                for name, alg in (("combined", iso.ISO_ALG_COMBINED), ("combined_bydim", iso.ISO_ALG_COMBINED_BYDIM),
                                  ("combined_staged", iso.ISO_ALG_COMBINED_STAGED), ("sx_fused", iso.ISO_ALG_SX_FUSED)):
                    wsb = iso.iso_workspace_bytes_v(icomm, iso.ISO_OP_ALLTOALL, alg, sizes)
                    iwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                    r = iso.iso_neighbor_alltoallv_init(isend, sizes, displs, ext, irecv, sizes, displs, ext,
                                                        iwork, icomm, alg)
                    ms = self.time_steps([r], ksteps, 3) / ksteps
                    extras[f"alltoallv_stencil_base64_{tag}{name}"] = rate([r], ms)
                    iso.iso_request_free(r)
                    del iwork
                del isend, irecv
            # the same blocks as one dense plane per neighbour (slot-major)
            pd, at = [], 0
            for sz in sizes:
                pd.append(at)
                at += -(-p * sz // 16) * 16
            psend = torch.empty(at, dtype=torch.uint8, device=dev).fill_(3)
            precv = torch.empty(at, dtype=torch.uint8, device=dev)
            for name, alg in (("combined", iso.ISO_ALG_COMBINED), ("sx_fused", iso.ISO_ALG_SX_FUSED)):
                wsb = iso.iso_workspace_bytes_v(icomm, iso.ISO_OP_ALLTOALL, alg, sizes)
                iwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                r = iso.iso_neighbor_alltoallv_init_layout(psend, sizes, pd, 0, precv, sizes, pd, 0,
                                                           iso.ISO_LAYOUT_SLOT_MAJOR, iwork, icomm, alg)
                ms = self.time_steps([r], ksteps, 3) / ksteps
                extras[f"alltoallv_stencil_base64_slot_major_{name}"] = rate([r], ms)
                iso.iso_request_free(r)
                del iwork
            del psend, precv
        # the same collectives on slot-major buffers ([s][p][m], one plane per neighbour): every
        # block-move is a dense stream on both sides, whatever m is
        for name, alg in (("combined", iso.ISO_ALG_COMBINED), ("combined_bydim", iso.ISO_ALG_COMBINED_BYDIM),
                          ("sx_fused", iso.ISO_ALG_SX_FUSED)):
            rs, keepalive = [], []
            for op in ops:
                if op == iso.ISO_OP_ALLTOALL:
                    sm_send = torch.empty((s, p, m), dtype=torch.uint8, device=dev).fill_(5)
                    init = iso.iso_neighbor_alltoall_init_layout
                else:
                    sm_send = self.bufs[op][0]
                    init = iso.iso_neighbor_allgather_init_layout
                sm_recv = torch.empty((s, p, m), dtype=torch.uint8, device=dev)
                wsb = iso.iso_workspace_bytes(comm, op, alg, m)
                sm_work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                rs.append(init(sm_send, sm_recv, m, iso.ISO_LAYOUT_SLOT_MAJOR, sm_work, comm, alg))
                keepalive += [sm_send, sm_recv, sm_work]
            ms = self.time_steps(rs, ksteps, 3) / ksteps
            extras[f"slot_major_{name}"] = rate(rs, ms, hbm_label=not (name.startswith("sx") and
                                                                       iso.ISO_OP_ALLGATHER in ops))
            for r in rs:
                iso.iso_request_free(r)
            del rs, keepalive
            torch.cuda.empty_cache()
        # the all-to-all with every rank's row padded by 128 bytes (the irregular interface's extents):
        # where the row size s*m is a multiple of 4 KiB, all blocks of a round sit at one offset
        # modulo 4 KiB; the padding spreads them
        if iso.ISO_OP_ALLTOALL in ops and p * (s * m + 128) <= (2 << 30):
            ext = s * m + 128
            sizes, displs = [m] * s, [i * m for i in range(s)]
            psend = torch.empty((p, ext), dtype=torch.uint8, device=dev).fill_(5)
            precv = torch.empty((p, ext), dtype=torch.uint8, device=dev)
            wsb = iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m)
            pwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
            r = iso.iso_neighbor_alltoallv_init(psend, sizes, displs, ext, precv, sizes, displs, ext, pwork, comm,
                                                iso.ISO_ALG_COMBINED)
            ms = self.time_steps([r], ksteps, 3) / ksteps
            extras["alltoall_rows_padded_128B_combined"] = rate([r], ms)
            iso.iso_request_free(r)
            del psend, precv, pwork
            torch.cuda.empty_cache()
        # the same torus taken as a box (no dimension wraps, Section 7): blocks whose source lies
        # outside stay untouched; moved bytes are nominal (every entry counted at every rank)
        if cfg is gen.get_config(2):
            mcomm = iso.iso_neighborhood_create_mesh(cfg.dims, (0,) * cfg.d, cfg.offsets)
            msend, mrecv = self.bufs[iso.ISO_OP_ALLTOALL]
            for name, alg in (("combined", iso.ISO_ALG_COMBINED), ("sx_fused", iso.ISO_ALG_SX_FUSED)):
                wsb = iso.iso_workspace_bytes(mcomm, iso.ISO_OP_ALLTOALL, alg, m)
                mwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                r = iso.iso_neighbor_alltoall_init(msend, mrecv, m, mwork, mcomm, alg)
                ms = self.time_steps([r], ksteps, 3) / ksteps
                d = rate([r], ms)
                extras[f"mesh_alltoall_{name}"] = {
                    "ms_per_step": d["ms_per_step"], "delivered_GBs_nominal": d["delivered_GBs"],
                    "moved_GBs_nominal": d["moved_GBs"], "frac_of_peak_nominal": d["frac_of_peak"],
                    "launches": d["launches"]}
                iso.iso_request_free(r)
                del mwork
        log(json.dumps(extras))
        return extras

    # -- CPU-oracle leg (the only part of this file that touches oracle/) --------------
    def cpu_leg(self, out, seconds):
        """(1) sampled ranks of the timed configuration against the oracle's source-rank table,
        (2) the oracle's C twin timed on the host cores, (3) its whole result against the GPU's."""
        from oracle import c_twin
        from oracle import iso_oracle as orc
        iso, torch, gen, np, args, cfg = self.iso, self.torch, self.gen, self.np, self.args, self.cfg
        p, s, m, dev, ops, slot = self.p, self.s, self.m, self.dev, self.ops, self.slot
        for op in ops:                                   # one more step of the timed requests, from scratch
            self.timed[op][1].fill_(0xEE)
        for r in self.reqs:
            iso.iso_start(r, self.stream)
        torch.cuda.synchronize()
        rng = np.random.default_rng(args.seed)
        sample = np.unique(rng.integers(0, p, size=min(p, 512)))
        src = torch.from_numpy(orc.source_ranks(cfg.dims, cfg.offsets, sample)).to(dev)
        slots = torch.arange(s, device=dev)[None, :]
        for op in ops:
            recv = self.timed[op][1].permute(1, 0, 2) if slot else self.timed[op][1]      # view as [p][s][m]
            if op == iso.ISO_OP_ALLTOALL:
                want = gen.block_bytes_torch(args.seed, src, slots, m, cfg.kind)
            else:
                want = gen.block_bytes_torch(args.seed ^ gen.ALLGATHER_TWEAK, src, torch.zeros_like(src), m, cfg.kind)
            if not bool(torch.equal(recv[torch.from_numpy(sample).to(dev)], want)):
                log("bench.py: RESULT MISMATCH against the oracle; aborting")
                sys.exit(3)
        host = {op: self.bufs[op][0].cpu().numpy() for op in ops}
        outs = {op: np.empty((p, s, m), np.uint8) for op in ops}
        times, used = [], 1
        t_begin = time.perf_counter()
        while True:
            t = time.perf_counter()
            for op in ops:
                fn = c_twin.alltoall if op == iso.ISO_OP_ALLTOALL else c_twin.allgather
                # threads: OpenMP's default the first time, then that same count explicitly (the
                # one-thread runs of an earlier workload leave the runtime's setting at 1)
                _, used = fn(cfg.dims, cfg.offsets, host[op], out=outs[op], threads=Bench.host_threads)
                Bench.host_threads = Bench.host_threads or int(used)
            times.append(time.perf_counter() - t)
            if (time.perf_counter() - t_begin > seconds and len(times) >= 3) or len(times) >= 5000:
                break
        for op in ops:                                   # the two sides agree on the whole buffer
            got = self.timed[op][1].permute(1, 0, 2) if slot else self.timed[op][1]
            if not np.array_equal(outs[op], got.cpu().numpy()):
                log("bench.py: GPU result differs from the C oracle")
                sys.exit(3)
        out["verified_against_oracle"] = True
        t_med = median(times[1:]) if len(times) > 1 else times[0]
        out["cpu_baseline"] = {
            "value": round(self.delivered / t_med / 1e9, 3), "unit": "GB/s", "cores": int(used), "kind": "oracle",
            "sample": f"whole workload ({'+'.join(cfg.ops)} of {cfg.name}, m={m}), {len(times)} repetitions, "
                      f"median; C twin of the oracle, OpenMP over ranks",
            "ms_per_step": round(t_med * 1e3, 3),
        }
        # the same oracle on one thread, and (small workloads only) its numpy form
        t1 = []
        for _ in range(3):
            t = time.perf_counter()
            for op in ops:
                fn = c_twin.alltoall if op == iso.ISO_OP_ALLTOALL else c_twin.allgather
                fn(cfg.dims, cfg.offsets, host[op], out=outs[op], threads=1)
            t1.append(time.perf_counter() - t)
            if sum(t1) > seconds / 2:
                break
        out["cpu_baseline"]["one_thread_GBs"] = round(self.delivered / median(t1) / 1e9, 3)
        if self.delivered <= (1 << 29):
            t = time.perf_counter()
            for op in ops:
                (orc.alltoall if op == iso.ISO_OP_ALLTOALL else orc.allgather)(cfg.dims, cfg.offsets, host[op])
            out["cpu_baseline"]["numpy_oracle_GBs"] = round(self.delivered / (time.perf_counter() - t) / 1e9, 3)

    def close(self):
        for r in self.reqs:
            self.iso.iso_request_free(r)
        self.reqs, self.bufs, self.timed, self.keep, self.arena = [], {}, {}, [], None   # Bench.arena stays
        self.torch.cuda.empty_cache()


def small_blocks(args, gen, iso):
    """Config 4 (64^3 torus, Moore radius 1, both collectives) at its small block sizes, where the
    paper's [p][s][m] rows make a round's writes sparse: the message-combining schedule as it is
    and regrouped for small blocks (--algorithm staged).  Both are priced on the same algorithmic
    bytes, those of the message-combining schedule: 2 * (V + W) * p * m per step."""
    import copy
    cfg = gen.get_config(4)
    out = {}
    for m in (16, 32, 64):
        row, algorithmic = {}, None
        for name in ("combined", "staged"):
            a = copy.copy(args)
            a.algorithm = name
            b = Bench(a, cfg, m)
            if name == "combined":
                algorithmic = b.moved
            ms = b.time_steps(b.reqs, args.steps, args.warmup) / args.steps
            row[name] = {"ms_per_step": round(ms, 5), "launches": b.launches,
                         "delivered_GBs": round(b.delivered / ms / 1e6, 1),
                         "algorithmic_GBs": round(algorithmic / ms / 1e6, 1),
                         "frac_of_peak": round(algorithmic / ms / 1e6 / HBM_PEAK_GBS, 4)}
            log(f"  small blocks: {cfg.name} m={m} {name}: {ms:.4f} ms/step, "
                f"{row[name]['frac_of_peak']:.3f} of peak on the schedule's {algorithmic / 1e6:.0f} MB")
            b.close()
        out[f"c4_m{m}"] = row
    return out


def main():
    args = parse()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (all p virtual ranks live in one device's HBM); "
            "--gpus must be 1.")
        sys.exit(2)

    import torch
    import iso_inputs as gen
    import paper_1606_07676_amd as iso

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    if args.small_sweep:
        small_sweep()
        return
    if args.setup_times:
        setup_times()
        return
    iso.load_library()
    torch.cuda.set_device(0)
    t_start = time.perf_counter()

    if args.config is not None:
        todo = [(gen.get_config(args.config), args.m)]
    else:
        # the workloads with blocks of 128 bytes and more, in ascending order of their footprint so
        # that each gets device memory that the larger ones have not been through; the last and
        # largest, config 5, is the headline
        todo = [(gen.get_config(2), None), (gen.get_config(3), None), (gen.get_config(4), None),
                (gen.get_config(5), None)]
    results = []
    head_idx = len(todo) - 1
    plain_run = not (args.mesh or args.irregular or args.pad)
    if plain_run:                                        # the run's arena, sized for its largest workload
        alg = {"combined": iso.ISO_ALG_COMBINED, "bydim": iso.ISO_ALG_COMBINED_BYDIM, "sx_fused": iso.ISO_ALG_SX_FUSED,
               "sx_rounds": iso.ISO_ALG_SX_ROUNDS, "onehop": iso.ISO_ALG_ONEHOP,
               "staged": iso.ISO_ALG_COMBINED_STAGED}[args.algorithm]
        need = 0
        for cfg, m_over in todo:
            comm = iso.iso_neighborhood_create(cfg.dims, cfg.offsets)
            ops = [iso.ISO_OP_ALLTOALL if o == "alltoall" else iso.ISO_OP_ALLGATHER for o in cfg.ops]
            need = max(need, Bench.arena_need(iso, comm, ops, cfg.p, cfg.s, m_over or cfg.m, args.layout == "slot", alg))
        # at least 8 GiB: the driver backs an allocation of several GiB with large physical blocks even
        # right after another process has freed tens of GB; a 2 GiB allocation made then can be scattered
        # (config 3 alone, after a config 5 process: 0.450 ms per step instead of 0.383)
        need = max(need, 8 << 30)
        Bench.arena = torch.empty(need + Bench.ALIGN, dtype=torch.uint8, device="cuda:0")
    for idx, (cfg, m_over) in enumerate(todo):
        b = Bench(args, cfg, m_over or cfg.m)
        res = b.run()
        if args.no_extras and args.copy_reference and idx == head_idx:
            res["copy_1GiB_GBs_read_plus_write"] = b.copy_reference_rate()
        # the comparison algorithms: on the one workload asked for, else on config 2 (small and quick)
        if not args.no_extras and b.plain and (args.config is not None or cfg is gen.get_config(2)) \
                and args.algorithm == "combined" and not args.graph:
            res["comparison"] = b.comparison()
        if not args.no_cpu_baseline and b.plain:
            b.cpu_leg(res, max(args.cpu_seconds, 10.0) if idx == head_idx else args.cpu_seconds)
        b.close()
        # (not when this process itself runs under the profiler, whose settings a child would inherit)
        profiled = any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ)
        if not (args.timed_only or args.no_live_traffic or profiled):
            # HBM traffic of this workload's launches, counted in child runs of this program
            counted = live_traffic(b.flags())
            if counted:
                roof = res["roofline"]
                roof["traffic"] = counted["bytes_per_launch"]
                roof["traffic_source"] = ("counted in this run: rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, around "
                                          "`bench.py " + " ".join(b.flags()) + " --steps 3 --warmup 1 --timed-only "
                                          "--no-cpu-baseline --no-extras --copy-reference`, scaled by the plain "
                                          "1 GiB copy of the same run")
                roof["traffic_fetched_written"] = [counted["fetched"], counted["written"]]
                roof["traffic_copy_scale"] = counted["copy_scale"]
                # the same fraction on the counted bytes (the s-exchange's allgather re-reads its send blocks
                # from the caches: there `frac`, on the requested bytes, is no HBM figure and this one is)
                roof["frac_on_counted_traffic"] = round(
                    counted["bytes_per_launch"] / (roof["avg_launch_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
                log(f"  HBM traffic per launch, counted: {counted['bytes_per_launch']} B "
                    f"({counted['bytes_per_launch'] / roof['algorithmic_bytes_per_launch']:.4f} x algorithmic)")
        results.append(res)
        log(f"  [{time.perf_counter() - t_start:.1f} s since start]")

    small = None
    if args.config is None and not args.no_extras and plain_run and args.algorithm == "combined" and not args.graph:
        small = small_blocks(args, gen, iso)
    head = results[head_idx]
    out = {
        "metric": METRIC, "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
    }
    out.update({k: v for k, v in head.items() if k not in ("value", "unit", "ms_per_step")})
    if len(results) > 1:
        # the other workloads of the same run: same protocol, own roofline and CPU baseline
        out["workloads"] = {r["config"]["profile_tag"]: {k: v for k, v in r.items() if k != "isolated_repetitions"}
                            for r in results}
        out["workloads"][head["config"]["profile_tag"]] = {"see": "top level of this line"}
    if small:
        out["small_blocks"] = small
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
