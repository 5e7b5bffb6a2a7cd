#!/usr/bin/env python3
"""Benchmark of the schedule-construction hot path on one MI355X.

Headline (`value`, `ms_per_step`, `roofline`): one step = the receive and send schedules of ALL ranks of the
largest configuration, p = 2^27 - 1 (q = 27): skips, baseblocks, range search, Alg. 4 for every rank, send rows by
neighbour look-up (Alg. 9's second loop); 29 GB of int32 tables are written per step.  The same JSON line carries
one record per baseline configuration under `configs`, each with its own roofline block and CPU-oracle baseline:
  C2  p = 2^20 + 1: schedules of all ranks, then their expansion for n = 256 blocks (one library call a step);
  C3  the headline itself;
  C4  p = 65 537, n = 4096: expansion of both tables (2.156 GB), through bcs_expand and through bcs_expand_ws;
  C5  2^20 seeded (p, r, root) triples of mixed q: receive rows, and send rows by Alg. 5.
Inputs are just (p, root, n) and the seeded triples: synthetic by construction.  Outputs are preallocated; nothing
crosses PCIe inside a timed region.  Kernel durations are device-side: the library gives every launch its own pair
of HIP events on the stream the kernel runs on, in a second timed region of the same steps.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

P = (1 << 20) + 1          # C2: non-power-of-two, q = 21
ROOT_RANK = 0
N_BLOCKS = 256             # C2's expansion; R = 276 rounds, x = 18 dummy rounds
P_C3 = (1 << 27) - 1       # C3, the headline: q = 27, 2 x 14.5 GB of tables
P_C4, N_C4 = 65537, 4096   # C4: q = 17, R = 4112 rounds, 2 x 1.078 GB of block tables
COUNT_C5 = 1 << 20         # C5: seeded triples, p log-uniform in [2, 2^31 - 1]

HBM_PEAK_GBS = 8000.0                       # MI355X HBM3E
INT_VALU_PEAK_GOPS = 256 * 4 * 16 * 2.4     # CUs x SIMDs x lanes x GHz = 39 321.6 G lane-ops/s (32-bit, full rate)


def csrc_digest():
    """Short hash of the kernel sources: counter figures below are tied to the sources they were profiled on."""
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2205_10072_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")):
            with open(os.path.join(d, name), "rb") as f:
                h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


# Counter figures that this run does not measure itself: rocprofv3 --pmc runs of this same file, summarised under
# profiles/ (FETCH_SIZE scaled x2.0 and WRITE_SIZE x1.0 by the 1 GiB copy calibration; KiB per dispatch).
# Key: (config, kernel).  `csrc`: csrc_digest() of the sources that were profiled; when the sources have changed
# since, the record is still printed but marked "stale": true, and a warning goes to stderr.
PROFILED = {
    "csrc": "f7b790bceae31f3a",
    "source": "profiles/c2_step_p1048577_n256.md, c3_sched_p134217727.md, c4_expand_p65537_n4096.md, c5_batch_2e20.md, "
              "allgather_tables_p1048577_n256.md",
    "counters": {
        # per dispatch: FETCH_SIZE / WRITE_SIZE in KiB as read, SQ_WAVES, SQ_INSTS_VALU / SQ_WAVES, SQ_INSTS_SALU / SQ_WAVES,
        # SQ_THREAD_CYCLES_VALU / SQ_ACTIVE_INST_VALU (lanes active per vector instruction, of 64)
        ("C3", "k_digits"): {'fetch_kib': 28, 'write_kib': 524288, 'waves': 2097152, 'valu_per_wave': 90.0, 'salu_per_wave': 25.5, 'active_lanes': 64.0},
        ("C3", "k_recv_uniform"): {'fetch_kib': 1048881, 'write_kib': 17694827, 'waves': 2097152, 'valu_per_wave': 915.4, 'salu_per_wave': 470.4, 'active_lanes': 63.9},
        ("C3", "k_send_lookup"): {'fetch_kib': 2031794, 'write_kib': 14155972, 'waves': 524288, 'valu_per_wave': 1002.0, 'salu_per_wave': 626.0, 'active_lanes': 64.0},
        ("C2", "k_digits"): {'fetch_kib': 31, 'write_kib': 4096, 'waves': 16388, 'valu_per_wave': 72.0, 'salu_per_wave': 25.5, 'active_lanes': 64.0},
        ("C2", "k_recv_uniform"): {'fetch_kib': 7278, 'write_kib': 132104, 'waves': 16388, 'valu_per_wave': 1055.4, 'salu_per_wave': 546.5, 'active_lanes': 63.7},
        ("C2", "k_send_lookup"): {'fetch_kib': 21069, 'write_kib': 110656, 'waves': 8193, 'valu_per_wave': 1126.9, 'salu_per_wave': 446.0, 'active_lanes': 63.2},
        ("C2", "k_expand_rows"): {'fetch_kib': 35345, 'write_kib': 1130584, 'waves': 1130500, 'valu_per_wave': 69.0, 'salu_per_wave': 9.0, 'active_lanes': 64.0},
        ("C4", "k_expand"): {'fetch_kib': 9004, 'write_kib': 1052688, 'waves': 263176, 'valu_per_wave': 258.5, 'salu_per_wave': 195.0, 'active_lanes': 63.3},
        ("C4", "k_rows_to_bytes"): {'fetch_kib': 2252, 'write_kib': 1280, 'waves': 5124, 'valu_per_wave': 50.0, 'salu_per_wave': 12.0, 'active_lanes': 64.0},
        ("C4", "k_expand_rows"): {'fetch_kib': 5135, 'write_kib': 1052924, 'waves': 1052692, 'valu_per_wave': 69.0, 'salu_per_wave': 9.0, 'active_lanes': 64.0},
        ("C5 recv_and_send", "k_batch"): {'fetch_kib': 9272, 'write_kib': 266240, 'waves': 16384, 'valu_per_wave': 6627.2, 'salu_per_wave': 2415.7, 'active_lanes': 63.5},
        ("C5 recv_only", "k_batch"): {'fetch_kib': 8406, 'write_kib': 135168, 'waves': 16384, 'valu_per_wave': 2813.4, 'salu_per_wave': 872.8, 'active_lanes': 63.8},
        ("AG", "k_allgather_tables"): {"fetch_kib": 41280, "write_kib": 2261412},
    },
}


def profiled(config, kernel, digest):
    ent = PROFILED["counters"].get((config, kernel))
    if ent is None:
        return None
    out = dict(ent)
    out["source"] = PROFILED["source"]
    out["profiled_at_csrc"] = PROFILED["csrc"]
    out["stale"] = PROFILED["csrc"] != digest
    return out


# ----------------------------------------------------------------------------------------------------------------
# One model of the vector-ALU work of the construction, used for every `alu` roofline below.  "Useful" lane-operations of one rank with its OWN q (a wave of the batch kernel runs
# its loops to the largest q among its lanes; that excess, the second-range branch of Alg. 4, the byte copies of a
# row and the sort of the batch kernel are not counted).  So `frac` = useful lane-ops/s / peak is at most the share
# of time the vector ALUs are busy, and falls below it by divergence and by everything that is not the method.
#   a row whose end points come from the table      the vector instructions k_recv_uniform executes (one rank a lane),
#                                                    SQ_INSTS_VALU x 64 of the counter profile of this configuration:
#                                                    the count depends on p (how many rounds a wave takes from the
#                                                    ranks' digits, how many from windows), so it is measured, not
#                                                    modelled; for this kernel `frac` is therefore its vector-ALU
#                                                    utilisation.  Without a profile entry: 55 ops for each of the first
#                                                    six rounds, 28 for each later one (17 for the rule, a window in one
#                                                    round of five), 80 of set-up
#   the batch kernel and Alg. 5, by the structure of the code (no counter fit):
#   a round of Alg. 4 on two digit masks            55 ops (window masks, candidate, bookkeeping)
#   set-up of a row                                 50 ops
#   a digit walk, one p per launch                  3 ops a level from level 7 up, 3 around the low-digit table read
#   a digit walk, p per lane (batch kernel)         4 ops a level from level 7 up, 10 around it
#   a row by walks                                  (q + 2) walks + 55 q + 50
#   a send row by Alg. 5: entry i = rounds 0..i of the to-neighbour's row: sum over i of (i + 3) walks (or table
#   reads) + 55 (i + 1) + 30
#   a send row as the batch kernel builds it: 30 ops an entry for the rule that takes an entry from the rank's own
#   digits, one digit walk a round for its case (c), and Alg. 5 for the entries the rule leaves: 0.23 an entry below
#   level 8 (1.8 a triple at C5, counted on the host build of the lane code), each the neighbour's rounds 0..k with
#   k + 3 walks, plus 40 ops to fetch the entry from the workgroup's list
# ----------------------------------------------------------------------------------------------------------------
def ops_walk(q, per_lane):
    return (4 * max(q - 7, 0) + 10) if per_lane else (3 * max(q - 7, 0) + 3)


def ops_recv_tabled(q):
    return 55 * min(q, 6) + 28 * max(q - 6, 0) + 80


def recv_tabled_model(config, p, q, digest):
    """("alu", lane-ops per launch, note) for k_recv_uniform over all p ranks: executed instructions from the profile
    of `config` if there is one, else the estimate above."""
    prof = profiled(config, "k_recv_uniform", digest)
    if prof is not None and "valu_per_wave" in prof:
        return ("alu", prof["valu_per_wave"] * prof["waves"] * prof["active_lanes"],
                "counters (executed vector lane-operations)" + (", of other sources: stale" if prof["stale"] else ""))
    return ("alu", ops_recv_tabled(q) * p, "model (estimate)")


def ops_recv_walks(q, per_lane, walks=None):
    walks = (q + 2) if walks is None else walks
    return walks * ops_walk(q, per_lane) + 55 * q + 50


def ops_send_alg5(q, per_lane, tabled=False):
    total = 0
    for i in range(q):
        total += (0 if tabled else (i + 3) * ops_walk(q, per_lane)) + 55 * (i + 1) + 30
    return total


def ops_send_direct(q, per_lane):
    w = ops_walk(q, per_lane)
    low = min(q, 8)
    entries = 0.23 * low                       # entries left to Alg. 5
    rounds = low / 2.0 + 0.5                   # their average k + 1
    return 30 * q + q * w + entries * (rounds * (55 + w) + 3 * w + 40)


def measure_valu_peak(torch, bcs):
    """Integer vector-ALU rate this GPU reaches on independent full-rate ops (G lane-ops/s)."""
    blocks, iters = 256 * 32, 4096
    sink = torch.empty(blocks * 256, dtype=torch.int32, device="cuda")
    bcs.bcs_valu_peak_launch(blocks, iters, sink)
    torch.cuda.synchronize()
    bcs.bcs_timing_begin()
    for _ in range(5):
        bcs.bcs_valu_peak_launch(blocks, iters, sink)
    torch.cuda.synchronize()
    ms, cnt = bcs.bcs_timing_end()["k_valu_peak"]
    ops = blocks * 256 * iters * bcs.VALU_PEAK_OPS_PER_ITER
    return ops / (ms / cnt) / 1e6


def cpu_info():
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"host_cpus": os.cpu_count(), "cpu_model": model}


def cpu_threads():
    return min(16, os.cpu_count() or 1)


def cpu_repeat(fn, budget_s):
    """Runs fn() until the budget is spent (at least once); returns (calls, seconds)."""
    done = 0
    t0 = time.perf_counter()
    while True:
        fn()
        done += 1
        el = time.perf_counter() - t0
        if el >= budget_s or done >= 1000:
            return done, el


def timed_steps(torch, bcs, step, steps, warmup):
    """`warmup` untimed steps, then two regions of exactly `steps` steps each: the plain launches (throughput), and
    the same steps with every launch carrying its own start/stop events (device time per kernel; the events cost a
    few microseconds a launch).  Returns (ms per step, ms per step with events, {kernel: (sum ms, launches, min, max)})."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    bcs.bcs_timing_begin()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    timing = bcs.bcs_timing_stats()
    return (t1 - t0) * 1e3 / steps, (t3 - t2) * 1e3 / steps, timing


def kernel_records(timing, steps, models, config, digest):
    """Per-kernel entries from the device-side durations.  `models`: {kernel: ("hbm", bytes per launch) or
    ("alu", useful lane-ops per launch)}; kernels without a model are listed with their times only."""
    out = {}
    for name, (ms, cnt, shortest, longest) in timing.items():
        avg_ms = ms / cnt
        ent = {"launches_per_step": cnt / steps, "avg_ms": avg_ms, "min_ms": shortest, "max_ms": longest,
               "ms_per_step": ms / steps}
        if name in models:
            bound, amount = models[name][:2]
            if len(models[name]) > 2:
                ent["ops_source"] = models[name][2]
            if len(models[name]) > 3:          # a second view: the bytes the kernel has to move, against the HBM peak
                ent["hbm_algorithmic_bytes"] = models[name][3]
                ent["hbm_frac"] = models[name][3] / avg_ms / 1e6 / HBM_PEAK_GBS
            if bound == "hbm":
                ent.update(bound="hbm", achieved=amount / avg_ms / 1e6, peak=HBM_PEAK_GBS, unit="GB/s",
                           algorithmic_bytes=amount)
            else:
                ent.update(bound="alu", achieved=amount / avg_ms / 1e6, peak=INT_VALU_PEAK_GOPS, unit="Gop/s",
                           useful_lane_ops=amount)
            ent["frac"] = ent["achieved"] / ent["peak"]
            prof = profiled(config, name, digest)
            ent["traffic"] = None
            if prof is not None:
                if "fetch_kib" in prof and "write_kib" in prof:
                    ent["traffic"] = (2 * prof["fetch_kib"] + prof["write_kib"]) * 1024
                if "valu_per_wave" in prof and "waves" in prof:
                    # share of the kernel's time that its vector instructions need on 1024 SIMDs at 4 cycles each
                    prof["valu_busy"] = prof["valu_per_wave"] * prof["waves"] * 4 / (1024 * 2.4e9) / (avg_ms * 1e-3)
                if "active_lanes" in prof:
                    prof["active_lane_fraction"] = prof["active_lanes"] / 64.0
                ent["counters"] = prof
        out[name] = ent
    return out


def dominant(kernels):
    name = max((k for k in kernels if "frac" in kernels[k]), key=lambda k: kernels[k]["ms_per_step"])
    return dict(kernels[name], kernel=name)


# ----------------------------------------------------------------------------------------------------------------
# The configurations
# ----------------------------------------------------------------------------------------------------------------
def run_c3(torch, bcs, steps, warmup, digest):
    p = P_C3
    q = bcs.bcs_q(p)
    recv = torch.empty((p, q), dtype=torch.int32, device="cuda")
    send = torch.empty((p, q), dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_sched_workspace_bytes(p, 0, p), dtype=torch.uint8, device="cuda")

    def step():
        bcs.bcs_sched_rooted_ws(p, ROOT_RANK, 0, p, recv, send, ws)

    ms, ms_ev, timing = timed_steps(torch, bcs, step, steps, warmup)
    # the receive kernel writes the int32 table and the slot-major bytes and reads the digit table (counted once)
    models = {"k_recv_uniform": recv_tabled_model("C3", p, q, digest) + (p * q * (4 + 1) + 4 * p,),
              "k_digits": ("alu", (ops_walk(q, False) + 12) * p),
              "k_send_lookup": ("hbm", p * q * (1 + 4))}          # reads the slot-major bytes, writes one int32 table
    kernels = kernel_records(timing, steps, models, "C3", digest)
    del recv, send, ws
    torch.cuda.empty_cache()
    return {"workload": "C3: p=2^27-1 (q=27), all ranks, root 0: int32 recv rows (Alg. 4) and send rows (look-up), "
                        "2 x 14.5 GB written per step", "p": p, "q": q,
            "steps": steps, "ms_per_step": ms, "ms_per_step_with_kernel_events": ms_ev,
            "value": p / (ms * 1e-3), "unit": "rank-schedules/s",
            "written_GBps": 2 * p * q * 4 / ms / 1e6,
            "roofline": dominant(kernels), "kernels": kernels}


def cpu_c3(budget_s):
    import oracle
    p, rows, threads = P_C3, 1 << 22, cpu_threads()
    calls, el = cpu_repeat(lambda: oracle.sched_range(p, r0=12345, r1=12345 + rows, want_send=False, threads=threads),
                           budget_s)
    return dict({"value": calls * rows / el, "unit": "rank-schedules/s", "cores": threads, "kind": "oracle",
                 "sample": "receive rows (Alg. 4) of %d x 2^22 ranks of p=2^27-1, from rank 12345, %.1f s; the send rows "
                           "by look-up are a gather of receive rows and are not in the sample" % (calls, el)},
                **cpu_info())


def run_c2(torch, bcs, steps, warmup, digest):
    q = bcs.bcs_q(P)
    R = bcs.bcs_rounds(P, N_BLOCKS)
    recv = torch.empty((P, q), dtype=torch.int32, device="cuda")
    send = torch.empty((P, q), dtype=torch.int32, device="cuda")
    rb = torch.empty((P, R), dtype=torch.int32, device="cuda")
    sb = torch.empty((P, R), dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_sched_expand_workspace_bytes(P, N_BLOCKS), dtype=torch.uint8, device="cuda")

    def step():
        # one call: receive rows, send rows by look-up, both block tables
        bcs.bcs_sched_expand_ws(P, ROOT_RANK, N_BLOCKS, recv, send, rb, sb, ws)

    ms, ms_ev, timing = timed_steps(torch, bcs, step, steps, warmup)
    models = {"k_expand_rows": ("hbm", P * R * 4), "k_expand": ("hbm", P * R * 4),
              "k_send_lookup": ("hbm", P * q * (1 + 4) + P * 24),   # slot-major bytes in; one table and its byte rows out
              "k_recv_uniform": recv_tabled_model("C2", P, q, digest),
              "k_digits": ("alu", (ops_walk(q, False) + 12) * P)}
    kernels = kernel_records(timing, steps, models, "C2", digest)
    construct_ms = sum(kernels[k]["ms_per_step"] for k in ("k_digits", "k_recv_uniform", "k_send_lookup") if k in kernels)
    exp = kernels.get("k_expand_rows") or kernels.get("k_expand")
    return {"workload": "C2: p=2^20+1 (q=21), all ranks, root 0: recv+send schedules, then expansion n=%d (R=%d "
                        "rounds), one call a step" % (N_BLOCKS, R), "p": P, "q": q, "n": N_BLOCKS, "rounds": R,
            "steps": steps, "ms_per_step": ms, "ms_per_step_with_kernel_events": ms_ev,
            "value": P / (ms * 1e-3), "unit": "rank-schedules/s (schedules and both block tables)",
            "construct_rank_schedules_per_s": P / (construct_ms * 1e-3),
            "expand_gbs": exp["achieved"] if exp else None,
            "roofline": dominant(kernels), "kernels": kernels}


def cpu_c2(budget_s):
    import oracle
    threads = cpu_threads()

    def one_step():
        recv, send = oracle.sched_range(P, root=ROOT_RANK, threads=threads)
        oracle.expand(P, N_BLOCKS, recv, threads=threads)
        oracle.expand(P, N_BLOCKS, send, threads=threads)

    calls, el = cpu_repeat(one_step, budget_s)
    return {"value": calls * P / el, "unit": "rank-schedules/s (schedules and both block tables)", "cores": threads,
            "kind": "oracle", "sample": "%d whole steps (all %d ranks: recv by Alg. 4, send by look-up, expansion "
                                        "n=%d), %.1f s" % (calls, P, N_BLOCKS, el)}


def run_c4(torch, bcs, steps, warmup, digest):
    p, n = P_C4, N_C4
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    recv = torch.empty((p, q), dtype=torch.int32, device="cuda")
    send = torch.empty((p, q), dtype=torch.int32, device="cuda")
    bcs.bcs_sched(p, 0, p, recv, send)
    rb = torch.empty((p, R), dtype=torch.int32, device="cuda")
    sb = torch.empty((p, R), dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_expand_workspace_bytes(p, n, 0, p), dtype=torch.uint8, device="cuda")
    nbytes = 2 * p * R * 4
    models = {"k_expand": ("hbm", p * R * 4), "k_expand_rows": ("hbm", p * R * 4),
              "k_rows_to_bytes": ("hbm", p * q * 4 + p * 24)}
    out = {"workload": "C4: p=65537 (q=17), n=4096 blocks (R=%d rounds): both (rank, round) -> block tables from "
                       "the schedule tables, 2 x %.3f GB written per step" % (R, p * R * 4 / 1e9),
           "p": p, "q": q, "n": n, "rounds": R, "steps": steps}
    for key, step in (("bcs_expand", lambda: bcs.bcs_expand(p, n, 0, p, recv, send, rb, sb)),
                      ("bcs_expand_ws", lambda: bcs.bcs_expand_ws(p, n, 0, p, recv, send, rb, sb, ws))):
        ms, ms_ev, timing = timed_steps(torch, bcs, step, steps, warmup)
        kernels = kernel_records(timing, steps, models, "C4", digest)
        dev_ms = sum(k["ms_per_step"] for k in kernels.values())
        out[key] = {"ms_per_step": ms, "ms_per_step_with_kernel_events": ms_ev, "device_ms_per_step": dev_ms,
                    "value": nbytes / ms / 1e6, "unit": "GB/s written (wall)",
                    "expand_gbs": nbytes / dev_ms / 1e6, "expand_frac": nbytes / dev_ms / 1e6 / HBM_PEAK_GBS,
                    "roofline": dominant(kernels), "kernels": kernels}
    out["roofline"] = out["bcs_expand_ws"]["roofline"]
    out["expand_gbs"] = out["bcs_expand_ws"]["expand_gbs"]
    out["expand_frac"] = out["bcs_expand_ws"]["expand_frac"]
    out["value"], out["unit"] = out["expand_gbs"], "GB/s written (device time, bcs_expand_ws)"
    out["ms_per_step"] = out["bcs_expand_ws"]["ms_per_step"]
    return out


def cpu_c4(budget_s):
    import oracle
    p, n, threads = P_C4, N_C4, cpu_threads()
    recv, send = oracle.sched_range(p, threads=threads)
    R = n - 1 + recv.shape[1]

    def both():
        oracle.expand(p, n, recv, threads=threads)
        oracle.expand(p, n, send, threads=threads)

    calls, el = cpu_repeat(both, budget_s)
    return {"value": calls * 2 * p * R * 4 / el / 1e9, "unit": "GB/s written", "cores": threads, "kind": "oracle",
            "sample": "%d whole expansions of both tables (p=65537, n=4096), %.1f s" % (calls, el)}


def run_c5(torch, bcs, steps, warmup, digest):
    import numpy as np
    from paper_2205_10072_amd import synth
    count = COUNT_C5
    hp, hr, hroot = synth.batch_triples(count)
    pp, rr, ro = (torch.from_numpy(a).cuda() for a in (hp, hr, hroot))
    brecv = torch.empty((count, 32), dtype=torch.int32, device="cuda")
    bsend = torch.empty((count, 32), dtype=torch.int32, device="cuda")
    qv = torch.empty(count, dtype=torch.int32, device="cuda")
    qs = np.array([int(v - 1).bit_length() for v in hp.tolist()], dtype=np.int64)
    hist = np.bincount(qs, minlength=32)
    ops_recv = sum(int(hist[q]) * ops_recv_walks(q, True) for q in range(32))
    ops_send = sum(int(hist[q]) * ops_send_direct(q, True) for q in range(32))
    out = {"workload": "C5: 2^20 seeded (p, r, root) triples, p log-uniform in [2, 2^31-1] (mixed q), rows of stride 32: "
                       "receive rows by Alg. 4, send rows without neighbour rows (entries from the rank's own digits where that is "
                       "exact, Alg. 5 for the rest)",
           "count": count, "steps": steps, "mean_q": float(qs.mean())}
    for key, step, ops in (("recv_and_send", lambda: bcs.bcs_sched_batch(pp, rr, ro, brecv, bsend, qv), ops_recv + ops_send),
                           ("recv_only", lambda: bcs.bcs_sched_batch(pp, rr, ro, brecv, None, qv), ops_recv)):
        ms, ms_ev, timing = timed_steps(torch, bcs, step, steps, warmup)
        # `frac` of this kernel: the vector instructions it executes (all 64 lanes active: the per-lane-p code is
        # branch-free in q) against the peak, i.e. its vector-ALU utilisation, from the counter profile of these
        # sources; when the sources have changed since the profile, the structural model of useful work instead
        prof = profiled("C5 " + key, "k_batch", digest)
        executed = None
        if prof is not None and not prof["stale"]:
            executed = prof["valu_per_wave"] * prof["waves"] * prof["active_lanes"]
        kernels = kernel_records(timing, steps, {"k_batch": ("alu", executed if executed else ops)}, "C5 " + key, digest)
        kernels["k_batch"]["ops_source"] = "counters (executed vector lane-operations)" if executed else "model (useful lane-operations)"
        kernels["k_batch"]["useful_lane_ops_model"] = ops
        kernels["k_batch"]["useful_frac_model"] = ops / kernels["k_batch"]["avg_ms"] / 1e6 / INT_VALU_PEAK_GOPS
        out[key] = {"ms_per_step": ms, "ms_per_step_with_kernel_events": ms_ev,
                    "value": count / (ms * 1e-3), "unit": "rank-schedules/s" if key == "recv_and_send" else "receive rows/s",
                    "useful_lane_ops_per_rank": ops / count, "roofline": dominant(kernels), "kernels": kernels}
    out["value"] = out["recv_and_send"]["value"]
    out["unit"] = "rank-schedules/s"
    out["ms_per_step"] = out["recv_and_send"]["ms_per_step"]
    out["roofline"] = out["recv_and_send"]["roofline"]
    return out


def cpu_c5(budget_s):
    import oracle
    from paper_2205_10072_amd import synth
    sample, threads = 1 << 17, cpu_threads()
    hp, hr, hroot = synth.batch_triples(COUNT_C5)
    calls, el = cpu_repeat(lambda: oracle.sched_batch(hp[:sample], hr[:sample], hroot[:sample], threads=threads), budget_s)
    return {"value": calls * sample / el, "unit": "rank-schedules/s", "cores": threads, "kind": "oracle",
            "sample": "%d x the first 2^17 of the 2^20 triples (recv by Alg. 4, send by Alg. 5), %.1f s" % (calls, el)}


AG_PROCESS = 777777        # the process whose tables are built in the allgather-tables workload


def bench_allgather_tables(torch, bcs, args):
    """Alg. 9 pack/unpack index tables of one process of a p = 2^20+1 allgather with n = 256 blocks per buffer."""
    q = bcs.bcs_q(P)
    R = bcs.bcs_rounds(P, N_BLOCKS)
    pack = torch.empty((R, P), dtype=torch.int32, device="cuda")
    unpack = torch.empty((R, P), dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_allgather_workspace_bytes(P), dtype=torch.uint8, device="cuda")

    def step():
        bcs.bcs_allgather_tables_ws(P, N_BLOCKS, AG_PROCESS, pack, unpack, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    steps = max(1, min(args.steps, 1000))
    # Two timed regions of exactly `steps` steps each.  The first is the plain path and gives the throughput; in the
    # second every launch carries its own start/stop events (which costs a few microseconds a launch, 4-5 % of a
    # step here) and gives the per-kernel device times for the rooflines.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    bcs.bcs_timing_begin()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timing = bcs.bcs_timing_end()
    ms_per_step_events = (t1 - t0) * 1e3 / steps
    ms, cnt = timing["k_allgather_tables"]
    avg_ms = ms / cnt
    nbytes = 2 * P * R * 4                                   # both tables, written once
    out = {
        "metric": "allgather pack/unpack index tables of one process, GB/s written vs HBM peak",
        "value": nbytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_with_kernel_events": ms_per_step_events,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": "p=2^20+1 processes, n=%d blocks per buffer, process %d: receive schedules of all "
                               "ranks (slot-major), then 2 tables of %d rounds x p roots" % (N_BLOCKS, AG_PROCESS, R),
                   "p": P, "q": q, "n": N_BLOCKS, "rounds": R},
        "roofline": {"kernel": "k_allgather_tables", "bound": "hbm", "achieved": nbytes / avg_ms / 1e6,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": nbytes / avg_ms / 1e6 / HBM_PEAK_GBS,
                     "traffic": None, "avg_ms": avg_ms},
        "kernels_ms": {k: v[0] / v[1] for k, v in timing.items()},
        "csrc": csrc_digest(),
    }
    prof = profiled("AG", "k_allgather_tables", out["csrc"])
    if prof is not None:
        out["roofline"]["traffic"] = (2 * prof["fetch_kib"] + prof["write_kib"]) * 1024
        out["roofline"]["counters"] = prof
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.allgather_tables(P, N_BLOCKS, AG_PROCESS)
        el = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": nbytes / el / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "one whole call (full schedule of all ranks, then both tables), %.1f s" % el}
    return out


def bench_partner_tables(torch, bcs, args):
    """Alg. 7 / Alg. 8: the to- and from-process tables of all p = 2^27-1 processes (q = 27), one kernel each."""
    p = 2**27 - 1
    q = bcs.bcs_q(p)
    to = torch.empty((p, q), dtype=torch.int32, device="cuda")
    frm = torch.empty((p, q), dtype=torch.int32, device="cuda")

    def step():
        bcs.bcs_allgather_partners(p, 0, p, to, frm)
        bcs.bcs_census_partners(p, 0, p, to, frm)

    steps = max(1, min(args.steps, 100))
    ms_per_step, _, timing = timed_steps(torch, bcs, step, steps, args.warmup)
    ms, cnt = timing["k_partner_tables"][:2]
    avg_ms = ms / cnt
    nbytes = 2 * p * q * 4                                   # per launch: both tables, written once
    out = {
        "metric": "partner tables of the regular allgather and the census for all processes, GB/s written vs HBM peak",
        "value": 2 * nbytes / (ms_per_step * 1e-3) / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": "p=2^27-1 processes (q=27): to/from tables of Alg. 7, then of Alg. 8, 4 tables of "
                               "p x q int32", "p": p, "q": q},
        "roofline": {"kernel": "k_partner_tables", "bound": "hbm", "achieved": nbytes / avg_ms / 1e6,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": nbytes / avg_ms / 1e6 / HBM_PEAK_GBS,
                     "traffic": None, "avg_ms": avg_ms},
        "csrc": csrc_digest(),
    }
    if not args.no_cpu_baseline:
        import oracle
        sample = 1 << 16
        t0 = time.perf_counter()
        for r in range(sample):
            oracle.allgather_plan(p, r)
            oracle.census_plan(p, r)
        el = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sample * q * 16 / el / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "the plans of %d processes, one call per process and collective (through "
                                         "ctypes), %.1f s" % (sample, el)}
    return out


def bench_shard(torch, bcs, args):
    """One GPU's share of C3 when the ranks are spread over eight GPUs with no exchange: ranks [0, p/8) of p = 2^27-1,
    receive rows and send rows without the other ranks' receive rows (entries from the ranks' own digits where the
    rule allows, Alg. 5 for the rest)."""
    p = P_C3
    q = bcs.bcs_q(p)
    r0, r1 = 0, (p + 7) // 8
    rows = r1 - r0
    recv = torch.empty((rows, q), dtype=torch.int32, device="cuda")
    send = torch.empty((rows, q), dtype=torch.int32, device="cuda")
    ws = torch.empty(max(1, bcs.bcs_sched_workspace_bytes(p, r0, r1)), dtype=torch.uint8, device="cuda")

    def step():
        bcs.bcs_sched_rooted_ws(p, ROOT_RANK, r0, r1, recv, send, ws)

    steps = max(1, min(args.steps, 100))
    ms, ms_ev, timing = timed_steps(torch, bcs, step, steps, args.warmup)
    kernels = {k: {"avg_ms": v[0] / v[1], "launches_per_step": v[1] / steps} for k, v in timing.items()}
    name = max(kernels, key=lambda k: kernels[k]["avg_ms"] * kernels[k]["launches_per_step"])
    out = {
        "metric": "rank-schedules constructed/s on one GPU's share of the ranks, no rows of other ranks",
        "value": rows / (ms * 1e-3), "unit": "rank-schedules/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms,
        "ms_per_step_with_kernel_events": ms_ev,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": "ranks [0, p/8) of p=2^27-1 (q=27): the digit masks of all ranks, receive rows of the share, "
                               "send rows of the share without the other ranks", "p": p, "q": q, "ranks": rows},
        "roofline": {"kernel": name, "bound": "alu", "achieved": None, "peak": INT_VALU_PEAK_GOPS, "unit": "Gop/s",
                     "frac": None, "traffic": None, "avg_ms": kernels[name]["avg_ms"],
                     "note": "no counter profile of this workload: times only"},
        "kernels_ms": {k: v["avg_ms"] for k, v in kernels.items()},
        "csrc": csrc_digest(),
    }
    if not args.no_cpu_baseline:
        import oracle
        sample, threads = 1 << 22, cpu_threads()
        t0 = time.perf_counter()
        oracle.sched_range(p, root=ROOT_RANK, r0=r0, r1=r0 + sample, threads=threads)
        el = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": sample / el, "unit": "rank-schedules/s", "cores": threads, "kind": "oracle",
                               "sample": "the first 2^22 ranks of the share: recv by Alg. 4, send by Alg. 5, %.1f s" % el}
    return out


PACK_P = 1152              # the paper's largest run: 36 nodes x 32 processes


def bench_pack_round(torch, bcs, args):
    """One round of Alg. 9's pack and unpack for process 0 of p = 1152, buffer sizes (r mod 3) * floor(m/p).
    Large case: m = 2^31 elements (8 GiB of buffers), n = 8 blocks, about 1 GiB moves per round.
    Paper-shaped case: m = 10^8 elements (400 MB), n = 1658 blocks (the paper's rule with G = 40): 241 KB."""
    import numpy as np
    from paper_2205_10072_amd import synth

    def setup(m, n):
        sizes, displs = synth.irregular_sizes(PACK_P, m)
        R = bcs.bcs_rounds(PACK_P, n)
        pack_t = torch.empty((R, PACK_P), dtype=torch.int32, device="cuda")
        unpack_t = torch.empty((R, PACK_P), dtype=torch.int32, device="cuda")
        bcs.bcs_allgather_tables(PACK_P, n, 0, pack_t, unpack_t)
        torch.cuda.synchronize()
        j = R // 2                                        # a round in the steady state: every root moves a block
        data = torch.empty(int(displs[-1]), dtype=torch.int32, device="cuda").random_(0, 1 << 30)
        d_displs = torch.from_numpy(displs).cuda()
        off = torch.empty(PACK_P + 1, dtype=torch.int64, device="cuda")
        ws = torch.empty(bcs.bcs_pack_workspace_bytes(PACK_P), dtype=torch.uint8, device="cuda")
        msg = torch.empty(int(sizes.max()) // n * PACK_P // 2 + 4 * PACK_P + 16, dtype=torch.int32, device="cuda")
        bcs.bcs_pack_round(n, pack_t[j], d_displs, data, msg, off, ws)
        torch.cuda.synchronize()
        length = int(off[PACK_P])
        assert 0 < length <= msg.numel()
        return dict(n=n, m=m, displs=displs, d_displs=d_displs, data=data, off=off, ws=ws, msg=msg, length=length,
                    pack_row=pack_t[j], unpack_row=pack_t[j])

    def run(c, steps, warmup):
        def step():
            bcs.bcs_pack_round(c["n"], c["pack_row"], c["d_displs"], c["data"], c["msg"], c["off"], c["ws"])
            bcs.bcs_unpack_round(c["n"], c["unpack_row"], c["d_displs"], c["data"], c["msg"], c["length"], c["off"],
                                 c["ws"])
        for _ in range(warmup):
            step()
        # a plain region for the time per round, then the same rounds with per-kernel events for the kernel times
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        bcs.bcs_timing_begin()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        timing = bcs.bcs_timing_end()
        return (t1 - t0) * 1e3 / steps, {k: v[0] / v[1] for k, v in timing.items()}

    steps = max(1, min(args.steps, 500))
    big = setup(1 << 31, 8)
    ms_big, k_big = run(big, steps, args.warmup)
    moved = 2 * 2 * big["length"] * 4                     # pack and unpack, each reads and writes the message once
    copy_bytes = 2 * big["length"] * 4
    out = {
        "metric": "pack + unpack of one allgather round on irregular buffers, GB/s moved vs HBM peak",
        "value": moved / (ms_big * 1e-3) / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_big,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": "p=1152, buffer sizes (r mod 3)*floor(m/p) with m=2^31 int32 elements, n=8 blocks, "
                               "process 0, a steady-state round: message of %d elements packed, then unpacked"
                               % big["length"], "p": PACK_P, "m": 1 << 31, "n": 8, "message_elements": big["length"]},
        "roofline": {"kernel": "k_pack_copy", "bound": "hbm", "achieved": copy_bytes / k_big["k_pack_copy"] / 1e6,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": copy_bytes / k_big["k_pack_copy"] / 1e6 / HBM_PEAK_GBS, "traffic": None,
                     "avg_ms": k_big["k_pack_copy"]},
        "kernels_ms": k_big,
    }
    del big
    torch.cuda.empty_cache()
    small = setup(100000000, 1658)
    ms_small, k_small = run(small, steps, args.warmup)
    out["paper_shaped"] = {"m": 100000000, "n": 1658, "message_bytes": small["length"] * 4,
                           "pack_plus_unpack_us": ms_small * 1e3, "kernels_ms": k_small}
    # the same round with the plans of all rounds made ahead in one launch (bcs_pack_plan_rounds): one kernel per
    # direction and round
    c = small
    R = bcs.bcs_rounds(PACK_P, c["n"])
    pack_t = torch.empty((R, PACK_P), dtype=torch.int32, device="cuda")
    unpack_t = torch.empty((R, PACK_P), dtype=torch.int32, device="cuda")
    bcs.bcs_allgather_tables(PACK_P, c["n"], 0, pack_t, unpack_t)
    offs = torch.empty((R, PACK_P + 1), dtype=torch.int64, device="cuda")
    srcs = torch.empty((R, PACK_P), dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    bcs.bcs_pack_plan_rounds(c["n"], pack_t, c["d_displs"], offs, srcs)
    torch.cuda.synchronize()
    plan_first_ms = (time.perf_counter() - t0) * 1e3
    bcs.bcs_timing_begin()
    for _ in range(5):
        bcs.bcs_pack_plan_rounds(c["n"], pack_t, c["d_displs"], offs, srcs)
    torch.cuda.synchronize()
    plan_ms = bcs.bcs_timing_end()["k_pack_plan"]
    j = R // 2

    def planned_round():
        bcs.bcs_pack_round_planned(offs[j], srcs[j], c["data"], c["msg"])
        bcs.bcs_unpack_round_planned(offs[j], srcs[j], c["data"], c["msg"], c["length"])

    # the binding's slicing of the plan rows is host work of the caller, so rows are taken once, as a real loop would
    oj, sj = offs[j], srcs[j]

    def planned_round_rows():
        bcs.bcs_pack_round_planned(oj, sj, c["data"], c["msg"])
        bcs.bcs_unpack_round_planned(oj, sj, c["data"], c["msg"], c["length"])

    for _ in range(args.warmup):
        planned_round_rows()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        planned_round_rows()
    torch.cuda.synchronize()
    planned_us = (time.perf_counter() - t0) * 1e6 / steps
    # the same rounds recorded into one HIP graph (consecutive rounds, each with its own plan rows): inside a graph
    # the kernels follow each other without the few microseconds that separate two launches of a stream
    g_rounds = min(256, R - j)
    g_rows = [(offs[j + i], srcs[j + i]) for i in range(g_rounds)]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for o, s in g_rows:
                bcs.bcs_pack_round_planned(o, s, c["data"], c["msg"])
                bcs.bcs_unpack_round_planned(o, s, c["data"], c["msg"], c["length"])
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        graph.replay()
    torch.cuda.synchronize()
    graph_us = (time.perf_counter() - t0) * 1e6 / (10 * g_rounds)
    del graph
    out["paper_shaped"]["planned"] = {"plan_all_rounds_ms": plan_ms[0] / plan_ms[1], "plan_first_call_ms": plan_first_ms,
                                      "rounds": R, "plan_bytes": int(offs.numel() + srcs.numel()) * 8,
                                      "pack_plus_unpack_us": planned_us,
                                      "pack_plus_unpack_us_in_hip_graph": graph_us, "graph_rounds": g_rounds}
    del pack_t, unpack_t, offs, srcs
    if not args.no_cpu_baseline:
        import oracle
        c = setup(1 << 28, 8)                             # an eighth of the large case keeps this to seconds
        h_idx = c["pack_row"].cpu().numpy()
        h_data = c["data"].cpu().numpy()
        t0 = time.perf_counter()
        msg, _ = oracle.pack_round(8, h_idx, c["displs"], h_data)
        oracle.unpack_round(8, h_idx, c["displs"], h_data, msg)
        el = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2 * 2 * len(msg) * 4 / el / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "same round at m=2^28 elements (message of %d elements), %.1f s" % (len(msg), el)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100,
                    help="timed steps of the headline configuration (C3); the other configurations time min(steps, 100)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", choices=["configs", "allgather-tables", "pack-round", "partner-tables", "shard"],
                    default="configs",
                    help="configs (default): the hot path on the baseline's configurations C2..C5, headline on C3.  "
                         "allgather-tables: the first widening, Alg. 9's pack/unpack index tables of one process, "
                         "reported as its own line.  pack-round: the second, packing and unpacking one round's message "
                         "on irregular buffers.  partner-tables: the to/from tables of Alg. 7 and Alg. 8 for all processes.  shard: one GPU's share of C3 (an eighth of the ranks) built without the other ranks")
    ap.add_argument("--only", default="C3,C2,C4,C5",
                    help="comma-separated subset of C2,C3,C4,C5 to run (for profiler runs; the headline needs C3)")
    ap.add_argument("--graph", action="store_true",
                    help="also record the C2 steps into one HIP graph and time its replay "
                         "(reported as ms_per_step_in_hip_graph in the C2 record)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies before the timed regions, so that a counter "
                         "profile of this command holds a kernel of known traffic to scale FETCH_SIZE/WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus %d is not supported (ranks shard trivially "
                 "over [r0, r1) with no exchange for receive rows)" % args.gpus)
    import torch
    import paper_2205_10072_amd as bcs
    bcs.lib()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if args.workload == "allgather-tables":
        print(json.dumps(bench_allgather_tables(torch, bcs, args)))
        return
    if args.workload == "pack-round":
        print(json.dumps(bench_pack_round(torch, bcs, args)))
        return
    if args.workload == "partner-tables":
        print(json.dumps(bench_partner_tables(torch, bcs, args)))
        return
    if args.workload == "shard":
        print(json.dumps(bench_shard(torch, bcs, args)))
        return
    only = [c.strip().upper() for c in args.only.split(",") if c.strip()]
    for c in only:
        if c not in ("C2", "C3", "C4", "C5"):
            sys.exit("bench.py: unknown configuration %r in --only" % c)
    digest = csrc_digest()
    if PROFILED["counters"] and PROFILED["csrc"] != digest:
        print("bench.py: kernel sources changed since the counter profiles were taken (%s -> %s): counter fields "
              "are marked stale" % (PROFILED["csrc"], digest), file=sys.stderr)
    if args.copy_calibration:
        a = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    steps = max(1, min(args.steps, 1000))
    sub_steps = min(steps, 100)
    sub_warm = min(args.warmup, 5)
    valu_peak_measured = measure_valu_peak(torch, bcs)
    runners = {"C3": lambda: run_c3(torch, bcs, steps, args.warmup, digest),
               "C2": lambda: run_c2(torch, bcs, sub_steps, sub_warm, digest),
               "C4": lambda: run_c4(torch, bcs, sub_steps, sub_warm, digest),
               "C5": lambda: run_c5(torch, bcs, sub_steps, sub_warm, digest)}
    cpu = {"C3": (cpu_c3, 7.0), "C2": (cpu_c2, 5.0), "C4": (cpu_c4, 4.0), "C5": (cpu_c5, 5.0)}
    configs = {}
    for c in only:
        configs[c] = runners[c]()
        torch.cuda.empty_cache()
    if args.graph and "C2" in configs:
        configs["C2"]["ms_per_step_in_hip_graph"] = c2_in_graph(torch, bcs, sub_steps)
    for rec in configs.values():                          # every alu roofline also against the measured ceiling
        for k in [rec.get("roofline")] + list(rec.get("kernels", {}).values()) + \
                 [sub.get("roofline") for sub in rec.values() if isinstance(sub, dict) and "roofline" in sub]:
            if k and k.get("bound") == "alu":
                k["peak_measured"] = valu_peak_measured
                k["frac_of_measured"] = k["achieved"] / valu_peak_measured
    if not args.no_cpu_baseline:
        for c in only:
            fn, budget = cpu[c]
            configs[c]["cpu_baseline"] = fn(budget)
    head = configs.get("C3") or configs[only[0]]
    out = {
        "metric": "rank-schedules constructed/s (int32, bit-exact) + expand GB/s vs HBM peak",
        "value": head["value"], "unit": head["unit"],
        "n_gpus": 1, "steps": head["steps"], "warmup": args.warmup if head is configs.get("C3") else sub_warm,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": head["workload"]},
        "roofline": head["roofline"],
        "csrc": digest,
    }
    if "C4" in configs:
        out["expand_gbs"] = configs["C4"]["expand_gbs"]
        out["expand_frac_of_hbm_peak"] = configs["C4"]["expand_frac"]
        out["expand_config"] = configs["C4"]["workload"]
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    out["configs"] = configs
    print(json.dumps(out))


def c2_in_graph(torch, bcs, steps):
    """The C2 steps as one HIP graph: inside a graph the kernels of consecutive steps follow each other without the
    few microseconds that separate two launches of a stream."""
    q = bcs.bcs_q(P)
    R = bcs.bcs_rounds(P, N_BLOCKS)
    recv = torch.empty((P, q), dtype=torch.int32, device="cuda")
    send = torch.empty((P, q), dtype=torch.int32, device="cuda")
    rb = torch.empty((P, R), dtype=torch.int32, device="cuda")
    sb = torch.empty((P, R), dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_sched_expand_workspace_bytes(P, N_BLOCKS), dtype=torch.uint8, device="cuda")
    bcs.bcs_sched_expand_ws(P, ROOT_RANK, N_BLOCKS, recv, send, rb, sb, ws)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(steps):
                bcs.bcs_sched_expand_ws(P, ROOT_RANK, N_BLOCKS, recv, send, rb, sb, ws)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


if __name__ == "__main__":
    main()
