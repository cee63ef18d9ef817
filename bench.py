#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: persistent isomorphic all-to-all and
allgather with the message-combining (torus-direct) schedule, one kernel per
round, on a synthetic workload held entirely in HBM.

One step = one iso_start of every collective the workload names (config 2:
all-to-all, then allgather), enqueued back to back on one stream.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line on stdout;
everything else goes to stderr.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak, GB/s


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="2", help="workload: 1..5 (default 2, the one the metric is quoted on)")
    ap.add_argument("--m", type=int, default=None, help="override the block size in bytes")
    ap.add_argument("--layout", choices=("rank", "slot"), default="rank",
                    help="buffers of the timed requests: rank = the paper's [p][s][m] (default), slot = [s][p][m]")
    ap.add_argument("--seed", type=int, default=2016)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the comparison algorithms and the copy ceiling")
    ap.add_argument("--copy-reference", action="store_true",
                    help="with --no-extras: still run the 1 GiB plain copy (calibration of the traffic counters)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--small-sweep", action="store_true",
                    help="instead of the benchmark: all-to-all on tori of about 500 processes (the paper's own "
                         "regime, Section 4), every algorithm, three block sizes; prints one JSON line")
    return ap.parse_args()


def recorded_traffic(cfg_name, m):
    """HBM bytes per launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE
    runs of this same command (counters cannot be read from inside the process).
    Only the workload the summary was taken on gets a value; anything else: None."""
    path = os.path.join(ROOT, "profiles", "shift_round_kernel_c2_hbm_traffic.txt")
    if not (cfg_name.startswith("c2_") and m == 256 and os.path.exists(path)):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch"):
            return int(line.split("=")[1])
    return None


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
            ("onehop", iso.ISO_ALG_ONEHOP), ("sx_rounds", iso.ISO_ALG_SX_ROUNDS), ("sx_fused", iso.ISO_ALG_SX_FUSED))
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
                for _ in range(10):
                    iso.iso_start(req, stream)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(200):
                    iso.iso_start(req, stream)
                e1.record(stream)
                torch.cuda.synchronize()
                row[an] = {"us": round(e0.elapsed_time(e1) / 200 * 1e3, 2),
                           "launches": iso.iso_request_info(req)["launches"]}
                iso.iso_request_free(req)
            log(row)
            rows.append(row)
    print(json.dumps({"small_sweep": rows}), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (all p virtual ranks live in one device's HBM); "
            "--gpus must be 1.")
        sys.exit(2)

    import numpy as np
    import torch
    import iso_inputs as gen
    import paper_1606_07676_amd as iso

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    if args.small_sweep:
        small_sweep()
        return
    iso.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = gen.get_config(args.config)
    m = args.m or cfg.m
    p, s = cfg.p, cfg.s
    K, W = args.steps, args.warmup
    stream = torch.cuda.current_stream()
    log(f"workload {cfg.name}: dims={cfg.dims} p={p} s={s} m={m} ops={cfg.ops}")

    # ---- set-up (host side of the hot path: neighbourhood, schedules, binding) ----
    t0 = time.perf_counter()
    comm = iso.iso_neighborhood_create(cfg.dims, cfg.offsets)
    t_create = (time.perf_counter() - t0) * 1e3
    cinfo = iso.iso_neighborhood_info(comm)

    ops = [iso.ISO_OP_ALLTOALL if o == "alltoall" else iso.ISO_OP_ALLGATHER for o in cfg.ops]
    op_name = {iso.ISO_OP_ALLTOALL: "alltoall", iso.ISO_OP_ALLGATHER: "allgather"}
    bufs = {}
    for op in ops:
        if op == iso.ISO_OP_ALLTOALL:
            send = gen.alltoall_send_torch(args.seed, p, s, m, cfg.kind, device=dev)
        else:
            send = gen.allgather_send_torch(args.seed, p, m, cfg.kind, device=dev)
        recv = torch.full((p, s, m), 0xEE, dtype=torch.uint8, device=dev)
        bufs[op] = (send, recv)
    # buffers of the timed requests; with --layout slot the same blocks as [s][p][m]
    slot = args.layout == "slot"
    timed = {}
    for op in ops:
        send, recv = bufs[op]
        if slot:
            tsend = send.permute(1, 0, 2).contiguous() if op == iso.ISO_OP_ALLTOALL else send
            timed[op] = (tsend, torch.full((s, p, m), 0xEE, dtype=torch.uint8, device=dev))
        else:
            timed[op] = (send, recv)

    def make_request(op, alg, timed_buffers=False):
        send, recv = timed[op] if timed_buffers else bufs[op]
        wsb = iso.iso_workspace_bytes(comm, op, alg, m)
        work = torch.empty(wsb, dtype=torch.uint8, device=dev) if wsb else None
        init = iso.iso_neighbor_alltoall_init_layout if op == iso.ISO_OP_ALLTOALL else \
            iso.iso_neighbor_allgather_init_layout
        layout = iso.ISO_LAYOUT_SLOT_MAJOR if (timed_buffers and slot) else iso.ISO_LAYOUT_RANK_MAJOR
        t = time.perf_counter()
        req = init(send, recv, m, layout, work, comm, alg)
        return req, (time.perf_counter() - t) * 1e3

    def time_steps(reqs, steps, warmup):
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

    reqs, t_init = [], []
    for op in ops:
        r, t = make_request(op, iso.ISO_ALG_COMBINED, timed_buffers=True)
        reqs.append(r)
        t_init.append(t)
    infos = [iso.iso_request_info(r) for r in reqs]
    delivered = sum(i["delivered_bytes"] for i in infos)
    moved = sum(i["bytes_read"] + i["bytes_written"] for i in infos)
    launches = sum(i["launches"] for i in infos)

    # ---- the timed region ------------------------------------------------------
    total_ms = time_steps(reqs, K, W)
    ms_per_step = total_ms / K
    value = delivered / (ms_per_step * 1e-3) / 1e9
    log(f"combined: {ms_per_step:.4f} ms/step, delivered {value:.1f} GB/s, moved "
        f"{moved / (ms_per_step * 1e-3) / 1e9:.1f} GB/s over {launches} launches")

    # ---- the paper's measurement protocol (Section 4): every repetition timed on its own
    # after a synchronisation, outliers outside [Q1 - 3 IQR, Q3 + 3 IQR] dropped, median kept
    reps = 100
    rep_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in rep_ev:
        torch.cuda.synchronize()
        a.record(stream)
        for r in reqs:
            iso.iso_start(r, stream)
        b.record(stream)
    torch.cuda.synchronize()
    rep_ms = sorted(a.elapsed_time(b) for a, b in rep_ev)
    q1, q3 = rep_ms[reps // 4], rep_ms[(3 * reps) // 4]
    kept = [t for t in rep_ms if q1 - 3 * (q3 - q1) <= t <= q3 + 3 * (q3 - q1)]
    protocol = {"repetitions": reps, "kept_after_tukey_3iqr": len(kept), "median_ms": round(median(kept), 5),
                "min_ms": round(kept[0], 5), "max_ms": round(kept[-1], 5),
                "delivered_GBs_at_median": round(delivered / median(kept) / 1e6, 1)}

    # ---- per-launch durations of the round kernel (HIP events on the launch stream) ----
    per_round = []
    ev_steps = max(1, min(K, 50))
    for r, inf in zip(reqs, infos):
        plan = iso.iso_request_plan(r)
        n = inf["launches"]
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
        for q in range(n):
            t_ms = median([evs[st][q][0].elapsed_time(evs[st][q][1]) for st in range(ev_steps)])
            nbytes = 2 * ks[q] * p * m
            per_round.append({"op": op_name[inf["op"]], "round": q, "dim": dims_[q], "k": ks[q],
                              "us": round(t_ms * 1e3, 2), "moved_GBs": round(nbytes / (t_ms * 1e-3) / 1e9, 1)})
    # Every launch of the step is the same kernel (shift_round_kernel, 16-byte units), so its
    # average launch duration over the timed region is region time / launches in the region.
    # This includes the gaps between back-to-back launches (the per-round event pairs above
    # additionally include the event markers themselves and are listed for orientation only).
    alg_bytes_per_launch = moved / launches
    avg_launch_ms = ms_per_step / launches
    achieved = alg_bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
    roofline = {
        "kernel": "shift_round_kernel<16B>",
        "bound": "hbm",
        "achieved": round(achieved, 1),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": None if slot else recorded_traffic(cfg.name, m),
        "algorithmic_bytes_per_launch": int(alg_bytes_per_launch),
        "avg_launch_us": round(avg_launch_ms * 1e3, 2),
        "launches_per_step": launches,
    }

    out = {
        "metric": "delivered GB/s (p*s*m bytes per collective / time) at 1 GPU; % of HBM peak",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u8",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: torus {'x'.join(map(str, cfg.dims))} (p={p}), s={s}, m={m} B, "
                        f"{'+'.join(cfg.ops)} per step, message-combining schedule, one kernel per round",
            "layout": "[s][p][m] (slot-major)" if slot else "[p][s][m] (rank-major, the paper's)",
            "algorithm": "combined (torus-direct)", "seed": args.seed,
            "rounds": cinfo["rounds"], "delivered_bytes_per_step": delivered, "moved_bytes_per_step": moved,
        },
        "verified_against_oracle": None,      # set by the CPU-oracle leg below
        "roofline": roofline,
        "isolated_repetitions": protocol,
        "per_round": per_round,
        "setup_ms": {"iso_neighborhood_create": round(t_create, 4),
                     **{f"iso_neighbor_{op_name[op]}_init": round(t, 4) for op, t in zip(ops, t_init)}},
    }

    def copy_reference_rate():
        """GB/s read + written by the library's plain copy kernel on 1 GiB: the ceiling, and the
        copy of known size that the HBM traffic counters are calibrated on."""
        nb = 1 << 30
        a = torch.empty(nb, dtype=torch.uint8, device=dev)
        b = torch.empty(nb, dtype=torch.uint8, device=dev)
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

    # ---- comparison algorithms and the copy ceiling (not part of `value`) -------
    if args.no_extras and args.copy_reference:
        out["copy_1GiB_GBs_read_plus_write"] = copy_reference_rate()
    if not args.no_extras:
        extras = {}
        ksteps = max(5, K // 4)
        for name, alg in (("combined_bydim", iso.ISO_ALG_COMBINED_BYDIM), ("sx_fused", iso.ISO_ALG_SX_FUSED),
                          ("sx_rounds", iso.ISO_ALG_SX_ROUNDS), ("onehop", iso.ISO_ALG_ONEHOP)):
            rs = [make_request(op, alg)[0] for op in ops]
            ms = time_steps(rs, ksteps, 3) / ksteps
            mv = sum(iso.iso_request_info(r)["bytes_read"] * 2 for r in rs)
            extras[name] = {"ms_per_step": round(ms, 5), "delivered_GBs": round(delivered / ms / 1e6, 1),
                            "moved_GBs": round(mv / ms / 1e6, 1),
                            "launches": sum(iso.iso_request_info(r)["launches"] for r in rs)}
            for r in rs:
                iso.iso_request_free(r)
        for op, r in zip(ops, reqs):
            ms = time_steps([r], ksteps, 3) / ksteps
            inf = iso.iso_request_info(r)
            extras[f"combined_{op_name[op]}_only"] = {
                "ms_per_step": round(ms, 5), "delivered_GBs": round(inf["delivered_bytes"] / ms / 1e6, 1),
                "moved_GBs": round(2 * inf["bytes_read"] / ms / 1e6, 1), "launches": inf["launches"]}
        for r in reqs:                                  # the same requests replayed as HIP graphs
            iso.iso_request_set_graph(r, True)
        ms = time_steps(reqs, ksteps, 3) / ksteps
        extras["combined_graph"] = {"ms_per_step": round(ms, 5), "delivered_GBs": round(delivered / ms / 1e6, 1),
                                    "moved_GBs": round(moved / ms / 1e6, 1), "launches": len(reqs)}
        for r in reqs:
            iso.iso_request_set_graph(r, False)
        extras["copy_1GiB_GBs_read_plus_write"] = copy_reference_rate()
        # irregular all-to-all in the shape of the paper's stencil experiment (Section 4): block of
        # neighbour i has base^(d - ||C^i||_1) bytes; same torus, Moore radius 1, base 64
        if cfg.d == 3 and args.config == "2":
            offs = gen.moore(3, 1)
            sizes = gen.stencil_block_sizes(offs, 64)
            icomm = iso.iso_neighborhood_create(cfg.dims, offs)
            # blocks at 16-byte aligned displacements, and packed back to back (rows of 25352 bytes)
            for tag, align in (("", 16), ("packed_", 1)):
                displs, ext = gen.packed_displacements(sizes, align)
                isend = torch.empty((p, ext), dtype=torch.uint8, device=dev).fill_(3)
                irecv = torch.empty((p, ext), dtype=torch.uint8, device=dev)
                for name, alg in (("combined", iso.ISO_ALG_COMBINED), ("sx_fused", iso.ISO_ALG_SX_FUSED)):
                    wsb = iso.iso_workspace_bytes_v(icomm, iso.ISO_OP_ALLTOALL, alg, sizes)
                    iwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                    r = iso.iso_neighbor_alltoallv_init(isend, sizes, displs, ext, irecv, sizes, displs, ext,
                                                        iwork, icomm, alg)
                    ms = time_steps([r], ksteps, 3) / ksteps
                    inf = iso.iso_request_info(r)
                    extras[f"alltoallv_stencil_base64_{tag}{name}"] = {
                        "ms_per_step": round(ms, 5), "delivered_GBs": round(inf["delivered_bytes"] / ms / 1e6, 1),
                        "moved_GBs": round(2 * inf["bytes_read"] / ms / 1e6, 1), "launches": inf["launches"]}
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
                ms = time_steps([r], ksteps, 3) / ksteps
                inf = iso.iso_request_info(r)
                extras[f"alltoallv_stencil_base64_slot_major_{name}"] = {
                    "ms_per_step": round(ms, 5), "delivered_GBs": round(inf["delivered_bytes"] / ms / 1e6, 1),
                    "moved_GBs": round(2 * inf["bytes_read"] / ms / 1e6, 1), "launches": inf["launches"]}
                iso.iso_request_free(r)
                del iwork
            del psend, precv
        # the same collectives on slot-major buffers ([s][p][m], one plane per neighbour): every
        # block-move is a dense stream on both sides, whatever m is
        sm_reqs = {}
        for name, alg in (("combined", iso.ISO_ALG_COMBINED), ("combined_bydim", iso.ISO_ALG_COMBINED_BYDIM),
                          ("sx_fused", iso.ISO_ALG_SX_FUSED)):
            rs, keepalive = [], []
            for op in ops:
                if op == iso.ISO_OP_ALLTOALL:
                    sm_send = torch.empty((s, p, m), dtype=torch.uint8, device=dev).fill_(5)
                    init = iso.iso_neighbor_alltoall_init_layout
                else:
                    sm_send = bufs[op][0]
                    init = iso.iso_neighbor_allgather_init_layout
                sm_recv = torch.empty((s, p, m), dtype=torch.uint8, device=dev)
                wsb = iso.iso_workspace_bytes(comm, op, alg, m)
                sm_work = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                rs.append(init(sm_send, sm_recv, m, iso.ISO_LAYOUT_SLOT_MAJOR, sm_work, comm, alg))
                keepalive += [sm_send, sm_recv, sm_work]
            ms = time_steps(rs, ksteps, 3) / ksteps
            mv = sum(iso.iso_request_info(r)["bytes_read"] * 2 for r in rs)
            extras[f"slot_major_{name}"] = {
                "ms_per_step": round(ms, 5), "delivered_GBs": round(delivered / ms / 1e6, 1),
                "moved_GBs": round(mv / ms / 1e6, 1), "frac_of_peak": round(mv / ms / 1e6 / HBM_PEAK_GBS, 4),
                "launches": sum(iso.iso_request_info(r)["launches"] for r in rs)}
            for r in rs:
                iso.iso_request_free(r)
            del rs, keepalive
            torch.cuda.empty_cache()
        # the all-to-all with every rank's row padded by 128 bytes (the irregular interface's extents):
        # where the row size s*m is a multiple of 4 KiB, all blocks of a round sit at one offset
        # modulo 4 KiB and load a fraction of the memory channels; the padding spreads them
        if iso.ISO_OP_ALLTOALL in ops and p * (s * m + 128) <= (2 << 30):
            ext = s * m + 128
            sizes, displs = [m] * s, [i * m for i in range(s)]
            psend = torch.empty((p, ext), dtype=torch.uint8, device=dev).fill_(5)
            precv = torch.empty((p, ext), dtype=torch.uint8, device=dev)
            wsb = iso.iso_workspace_bytes(comm, iso.ISO_OP_ALLTOALL, iso.ISO_ALG_COMBINED, m)
            pwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
            r = iso.iso_neighbor_alltoallv_init(psend, sizes, displs, ext, precv, sizes, displs, ext, pwork, comm,
                                                iso.ISO_ALG_COMBINED)
            ms = time_steps([r], ksteps, 3) / ksteps
            inf = iso.iso_request_info(r)
            extras["alltoall_rows_padded_128B_combined"] = {
                "ms_per_step": round(ms, 5), "delivered_GBs": round(inf["delivered_bytes"] / ms / 1e6, 1),
                "moved_GBs": round(2 * inf["bytes_read"] / ms / 1e6, 1),
                "frac_of_peak": round(2 * inf["bytes_read"] / ms / 1e6 / HBM_PEAK_GBS, 4), "launches": inf["launches"]}
            iso.iso_request_free(r)
            del psend, precv, pwork
            torch.cuda.empty_cache()
        # the same torus taken as a box (no dimension wraps, Section 7): blocks whose source lies
        # outside stay untouched; moved bytes are nominal (every entry counted at every rank)
        if args.config == "2":
            mcomm = iso.iso_neighborhood_create_mesh(cfg.dims, (0,) * cfg.d, cfg.offsets)
            msend, mrecv = bufs[iso.ISO_OP_ALLTOALL]
            for name, alg in (("combined", iso.ISO_ALG_COMBINED), ("sx_fused", iso.ISO_ALG_SX_FUSED)):
                wsb = iso.iso_workspace_bytes(mcomm, iso.ISO_OP_ALLTOALL, alg, m)
                mwork = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
                r = iso.iso_neighbor_alltoall_init(msend, mrecv, m, mwork, mcomm, alg)
                ms = time_steps([r], ksteps, 3) / ksteps
                inf = iso.iso_request_info(r)
                extras[f"mesh_alltoall_{name}"] = {
                    "ms_per_step": round(ms, 5), "delivered_GBs_nominal": round(inf["delivered_bytes"] / ms / 1e6, 1),
                    "moved_GBs_nominal": round(2 * inf["bytes_read"] / ms / 1e6, 1), "launches": inf["launches"]}
                iso.iso_request_free(r)
                del mwork
        out["comparison"] = extras
        log(json.dumps(extras))

    # ---- CPU-oracle leg (the only part of this file that touches oracle/) --------
    # (1) sampled ranks of the timed configuration against the oracle's source-rank table,
    # (2) the oracle's C twin timed on the host cores, (3) its whole result against the GPU's.
    if not args.no_cpu_baseline:
        from oracle import c_twin
        from oracle import iso_oracle as orc
        for op in ops:                                   # one more step of the timed requests, from scratch
            timed[op][1].fill_(0xEE)
        for r in reqs:
            iso.iso_start(r, stream)
        torch.cuda.synchronize()
        rng = np.random.default_rng(args.seed)
        sample = np.unique(rng.integers(0, p, size=min(p, 512)))
        src = torch.from_numpy(orc.source_ranks(cfg.dims, cfg.offsets, sample)).to(dev)
        slots = torch.arange(s, device=dev)[None, :]
        for op in ops:
            recv = timed[op][1].permute(1, 0, 2) if slot else timed[op][1]      # view as [p][s][m]
            if op == iso.ISO_OP_ALLTOALL:
                want = gen.block_bytes_torch(args.seed, src, slots, m, cfg.kind)
            else:
                want = gen.block_bytes_torch(args.seed ^ gen.ALLGATHER_TWEAK, src, torch.zeros_like(src), m, cfg.kind)
            if not bool(torch.equal(recv[torch.from_numpy(sample).to(dev)], want)):
                log("bench.py: RESULT MISMATCH against the oracle; aborting")
                sys.exit(3)
        host = {}
        for op in ops:
            host[op] = bufs[op][0].cpu().numpy()
        outs = {op: np.empty((p, s, m), np.uint8) for op in ops}
        times, used = [], 1
        t_begin = time.perf_counter()
        while True:
            t = time.perf_counter()
            for op in ops:
                fn = c_twin.alltoall if op == iso.ISO_OP_ALLTOALL else c_twin.allgather
                _, used = fn(cfg.dims, cfg.offsets, host[op], out=outs[op])
            times.append(time.perf_counter() - t)
            if (time.perf_counter() - t_begin > args.cpu_seconds and len(times) >= 3) or len(times) >= 5000:
                break
        for op in ops:                                   # the two sides agree on the whole buffer
            got = timed[op][1].permute(1, 0, 2) if slot else timed[op][1]
            if not np.array_equal(outs[op], got.cpu().numpy()):
                log("bench.py: GPU result differs from the C oracle")
                sys.exit(3)
        out["verified_against_oracle"] = True
        t_med = median(times[1:]) if len(times) > 1 else times[0]
        out["cpu_baseline"] = {
            "value": round(delivered / t_med / 1e9, 3), "unit": "GB/s", "cores": int(used), "kind": "oracle",
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
            if sum(t1) > args.cpu_seconds:
                break
        out["cpu_baseline"]["one_thread_GBs"] = round(delivered / median(t1) / 1e9, 3)
        if delivered <= (1 << 29):
            t = time.perf_counter()
            for op in ops:
                (orc.alltoall if op == iso.ISO_OP_ALLTOALL else orc.allgather)(cfg.dims, cfg.offsets, host[op])
            out["cpu_baseline"]["numpy_oracle_GBs"] = round(delivered / (time.perf_counter() - t) / 1e9, 3)

    for r in reqs:
        iso.iso_request_free(r)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
