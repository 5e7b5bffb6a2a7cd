#!/usr/bin/env python3
"""Benchmark of the schedule-construction hot path on one MI355X.

One step = one pass of the whole path over one batch: receive and send schedules of all
p = 2^20 + 1 ranks (skips, baseblocks, range search, Alg. 4, send by neighbour look-up,
root rotation) followed by their expansion into (rank, round) -> block tables for n = 256
blocks (Alg. 6 index arithmetic).  Inputs are just (p, root, n): synthetic by construction.
Outputs are preallocated; nothing crosses PCIe inside the timed region.

Prints ONE JSON line: rank-schedules per second over the whole step, the roofline of the
kernel that takes most of the step (plus one entry per kernel), the expansion's write rate,
and the CPU oracle timed on the host cores next to it (a baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

P = (1 << 20) + 1          # the headline configuration: non-power-of-two, q = 21
ROOT_RANK = 0
N_BLOCKS = 256             # expansion of the same tables; R = 276 rounds, x = 18 dummy rounds

HBM_PEAK_GBS = 8000.0                       # MI355X HBM3E
INT_VALU_PEAK_GOPS = 256 * 4 * 16 * 2.4     # CUs x SIMDs x lanes x GHz = 39 321.6 G lane-ops/s (32-bit, full rate)


# HBM bytes per launch at this workload, from the rocprofv3 counter runs summarised in
# profiles/bench_c2_kernels.md (FETCH_SIZE scaled x2.0, WRITE_SIZE x1.0 by the 1 GiB copy calibration).
PROFILED_TRAFFIC_BYTES = {
    "k_expand_rows": (2 * 35344 + 1130583) * 1024,
    "k_recv_uniform": (2 * 11364 + 132103) * 1024,
    "k_send_lookup": (2 * 15914 + 110592) * 1024,
    "k_digits": (2 * 32 + 4096) * 1024,
}


# SQ_INSTS_VALU / SQ_WAVES and SQ_THREAD_CYCLES_VALU / SQ_ACTIVE_INST_VALU of k_recv_uniform at this workload, from the
# same profile: vector instructions a wave (one rank a lane) and lanes active per vector instruction.
PROFILED_VALU_PER_WAVE = 1275
PROFILED_ACTIVE_LANES = 64.0


def digit_walks_per_rank(p, skips):
    """Digit walks k_recv_uniform runs per rank at root 0, averaged over all ranks: one for the rank itself, one for
    the first window's upper end, and one per round n = 1..q-1 in which some lane of the wave lacks skips[n] among
    its digits (when the whole wave has it, the end point's digits are the rank's with that digit taken out; the last
    round's end point is the rank itself).  Counted here by doing the greedy sums (Alg. 2's walk) of all ranks with
    numpy, 64 consecutive ranks a wave as the kernel lays them out."""
    import numpy as np
    q = len(skips) - 1
    rest = np.arange(p, dtype=np.int64)
    digits = np.zeros(p, dtype=np.int64)
    for k in range(q - 1, -1, -1):
        take = rest >= skips[k]
        rest -= take * skips[k]
        digits |= take.astype(np.int64) << k
    waves = -(-p // 64)
    padded = np.zeros(waves * 64, dtype=np.int64)        # idle lanes replay rank 0, which has no digits
    padded[:p] = digits
    shared = np.bitwise_and.reduce(padded.reshape(waves, 64), axis=1)
    direct = np.zeros(waves, dtype=np.int64)
    for n in range(1, q):
        direct += (shared >> n) & 1
    return float(2 + (q - 1) - direct.mean())


def valu_ops_per_rank_tabled(q):
    """The same row when the digit masks of all ranks are in a table (launches over all ranks):
    55 ops a round, which include the read of the round's end point, and 50 of set-up."""
    return 55 * q + 50


def valu_ops_per_rank(q, walks):
    """Vector-ALU lane-operations one receive row costs on the main path of k_recv_uniform, counted from its ISA:
    `walks` digit walks of 3 ops a level for the levels from 7 up and 3 ops around the table read that stands for
    the seven levels below, 55 ops of window logic and bookkeeping a round, 50 of set-up.
    The wave-uniform branch for Alg. 4's second range is extra work and not counted."""
    return (3 * max(q - 7, 0) + 3) * walks + 55 * q + 50


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


def cpu_baseline(budget_s=10.0):
    """The oracle, as it stands, on the host cores: whole steps of the same workload until the budget is spent;
    then one more step on a single thread."""
    import oracle

    def one_step(threads):
        recv, send = oracle.sched_range(P, root=ROOT_RANK, threads=threads)
        oracle.expand(P, N_BLOCKS, recv, threads=threads)
        oracle.expand(P, N_BLOCKS, send, threads=threads)

    threads = min(16, os.cpu_count() or 1)
    done = 0
    t0 = time.perf_counter()
    while True:
        one_step(threads)
        done += 1
        el = time.perf_counter() - t0
        if el >= budget_s or done >= 1000:
            break
    t1 = time.perf_counter()
    one_step(1)
    single = time.perf_counter() - t1
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {"value": done * P / el, "unit": "rank-schedules/s", "cores": threads, "kind": "oracle",
            "sample": "%d whole steps (all %d ranks: recv by Alg. 4, send by look-up, expansion n=%d), %.1f s"
                      % (done, P, N_BLOCKS, el),
            "single_thread_value": P / single, "host_cpus": os.cpu_count(), "cpu_model": model}


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
                     # from profiles/allgather_tables_p1048577_n256.md (FETCH_SIZE x2.0, WRITE_SIZE x1.0)
                     "traffic": (2 * 41280 + 2261412) * 1024, "avg_ms": avg_ms},
        "kernels_ms": {k: v[0] / v[1] for k, v in timing.items()},
    }
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.allgather_tables(P, N_BLOCKS, AG_PROCESS)
        el = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": nbytes / el / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "one whole call (full schedule of all ranks, then both tables), %.1f s" % el}
    return out


def bench_configs(torch, bcs, args):
    """Per-call device time of the baseline's other configurations (each parity-tested in tests/)."""
    from paper_2205_10072_amd import synth
    reps = max(3, min(args.steps, 20))

    def kernels(fn):
        fn()
        torch.cuda.synchronize()
        bcs.bcs_timing_begin()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        t = bcs.bcs_timing_end()
        return {k: v[0] / v[1] * (v[1] / reps) for k, v in t.items()}      # ms per call, summed over its launches

    out = {"metric": "per-call device time of the other baseline configurations", "unit": "ms", "n_gpus": 1,
           "steps": reps, "data": "synthetic", "dtype": "int32", "results": {}}
    res = out["results"]
    # C3: p = 2^27 - 1, all ranks, recv + send by look-up
    p = (1 << 27) - 1
    q = bcs.bcs_q(p)
    recv = torch.empty((p, q), dtype=torch.int32, device="cuda")
    send = torch.empty((p, q), dtype=torch.int32, device="cuda")
    k = kernels(lambda: bcs.bcs_sched(p, 0, p, recv, send))
    ms = sum(k.values())
    res["C3 p=2^27-1 all ranks recv+send"] = {"ms": ms, "kernels_ms": k, "rank_schedules_per_s": p / ms * 1e3,
                                              "written_GBps": 2 * p * q * 4 / ms / 1e6}
    # partial range of the same p: send rows by Alg. 5
    n_part = 1 << 20
    k = kernels(lambda: bcs.bcs_sched(p, 12345, 12345 + n_part, recv[:n_part], send[:n_part]))
    ms = sum(k.values())
    res["p=2^27-1, 2^20 ranks, send by Alg. 5"] = {"ms": ms, "kernels_ms": k, "rank_schedules_per_s": n_part / ms * 1e3}
    del recv, send
    bcs.bcs_release()
    torch.cuda.empty_cache()
    # C2 partial
    p = (1 << 20) + 1
    q = bcs.bcs_q(p)
    recv = torch.empty((n_part, q), dtype=torch.int32, device="cuda")
    send = torch.empty((n_part, q), dtype=torch.int32, device="cuda")
    k = kernels(lambda: bcs.bcs_sched(p, 1, 1 + n_part, recv, send))
    ms = sum(k.values())
    res["p=2^20+1, 2^20 ranks, send by Alg. 5"] = {"ms": ms, "kernels_ms": k, "rank_schedules_per_s": n_part / ms * 1e3}
    # short rows, all four tables of all ranks: one call (fused kernels) against the separate calls
    n = 64
    R = bcs.bcs_rounds(p, n)
    recv = torch.empty((p, q), dtype=torch.int32, device="cuda")
    send = torch.empty((p, q), dtype=torch.int32, device="cuda")
    rb = torch.empty((p, R), dtype=torch.int32, device="cuda")
    sb = torch.empty((p, R), dtype=torch.int32, device="cuda")
    ws = torch.empty(bcs.bcs_sched_workspace_bytes(p, 0, p), dtype=torch.uint8, device="cuda")
    k = kernels(lambda: bcs.bcs_sched_expand_ws(p, 0, n, recv, send, rb, sb, ws))
    ms = sum(k.values())
    res["p=2^20+1 n=64 schedules+tables, one call"] = {"ms": ms, "kernels_ms": k, "rank_schedules_per_s": p / ms * 1e3}
    k = kernels(lambda: (bcs.bcs_sched_rooted_ws(p, 0, 0, p, recv, send, ws), bcs.bcs_expand(p, n, 0, p, recv, send, rb, sb)))
    ms = sum(k.values())
    res["p=2^20+1 n=64 schedules+tables, separate calls"] = {"ms": ms, "kernels_ms": k,
                                                             "rank_schedules_per_s": p / ms * 1e3}
    del rb, sb, ws
    # C4: expansion p = 65537, n = 4096
    p, n = 65537, 4096
    q, R = bcs.bcs_q(p), bcs.bcs_rounds(p, n)
    recv = torch.empty((p, q), dtype=torch.int32, device="cuda")
    send = torch.empty((p, q), dtype=torch.int32, device="cuda")
    bcs.bcs_sched(p, 0, p, recv, send)
    rb = torch.empty((p, R), dtype=torch.int32, device="cuda")
    sb = torch.empty((p, R), dtype=torch.int32, device="cuda")
    k = kernels(lambda: bcs.bcs_expand(p, n, 0, p, recv, send, rb, sb))
    ms = sum(k.values())
    res["C4 expand p=65537 n=4096"] = {"ms": ms, "kernels_ms": k, "written_GBps": 2 * p * R * 4 / ms / 1e6,
                                      "frac_of_hbm_peak": 2 * p * R * 4 / ms / 1e6 / HBM_PEAK_GBS}
    ws = torch.empty(bcs.bcs_expand_workspace_bytes(p, n, 0, p), dtype=torch.uint8, device="cuda")
    k = kernels(lambda: bcs.bcs_expand_ws(p, n, 0, p, recv, send, rb, sb, ws))
    ms = sum(k.values())
    res["C4 expand p=65537 n=4096, with workspace"] = {"ms": ms, "kernels_ms": k, "written_GBps": 2 * p * R * 4 / ms / 1e6,
                                                      "frac_of_hbm_peak": 2 * p * R * 4 / ms / 1e6 / HBM_PEAK_GBS}
    del ws
    del rb, sb
    # C5: 2^20 seeded triples, mixed q
    count = 1 << 20
    pp, rr, ro = (torch.from_numpy(a).cuda() for a in synth.batch_triples(count))
    brecv = torch.empty((count, 32), dtype=torch.int32, device="cuda")
    bsend = torch.empty((count, 32), dtype=torch.int32, device="cuda")
    qv = torch.empty(count, dtype=torch.int32, device="cuda")
    k = kernels(lambda: bcs.bcs_sched_batch(pp, rr, ro, brecv, bsend, qv))
    ms = sum(k.values())
    res["C5 batch 2^20 triples recv+send"] = {"ms": ms, "kernels_ms": k, "rank_schedules_per_s": count / ms * 1e3}
    k = kernels(lambda: bcs.bcs_sched_batch(pp, rr, ro, brecv, None, qv))
    res["C5 batch 2^20 triples recv only"] = {"ms": sum(k.values()), "rank_schedules_per_s": count / sum(k.values()) * 1e3}
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
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", choices=["step", "allgather-tables", "pack-round", "configs"], default="step",
                    help="step (default): the hot path this benchmark is about.  allgather-tables: the first widening, "
                         "Alg. 9's pack/unpack index tables of one process, reported as its own line.  pack-round: the second, "
                         "packing and unpacking one round's message on irregular buffers.  configs: the other "
                         "configurations of the baseline (largest p, expansion at p=65537, irregular batch, partial "
                         "ranges), one line of per-call timings")
    ap.add_argument("--graph", action="store_true",
                    help="step workload only: also record the timed steps into one HIP graph and time its replay "
                         "(reported as ms_per_step_in_hip_graph; `value` stays the plain launches)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies before the timed region, so that a counter "
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
    if args.workload == "configs":
        print(json.dumps(bench_configs(torch, bcs, args)))
        return
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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        a = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    valu_peak_measured = measure_valu_peak(torch, bcs)
    tabled = True                                        # all ranks: receive rows read the digit masks k_digits leaves
    walks = 1.0 if tabled else digit_walks_per_rank(P, bcs.bcs_skips(P))
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
    timing = bcs.bcs_timing_stats()
    ms_per_step_events = (t1 - t0) * 1e3 / steps

    ms_per_step_graph = None
    if args.graph:
        # the same steps as one HIP graph: inside a graph the kernels of consecutive steps follow each other without
        # the few microseconds that separate two launches of a stream
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(steps):
                    step()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / steps

    # per-kernel rooflines from the device-side durations of the timed region
    kernels = {}
    for name, (ms, cnt, shortest, longest) in timing.items():
        avg_ms = ms / cnt
        ent = {"launches_per_step": cnt / steps, "avg_ms": avg_ms, "min_ms": shortest, "max_ms": longest,
               "ms_per_step": ms / steps}
        if name in ("k_expand", "k_expand_rows"):
            nbytes = P * R * 4                                  # one table per launch, written once
            ent.update(bound="hbm", achieved=nbytes / avg_ms / 1e6, peak=HBM_PEAK_GBS, unit="GB/s")
        elif name == "k_send_lookup":
            nbytes = P * q * (1 + 4) + P * 24                   # read the slot-major bytes, write one table and its byte rows
            ent.update(bound="hbm", achieved=nbytes / avg_ms / 1e6, peak=HBM_PEAK_GBS, unit="GB/s")
        elif name == "k_recv_uniform":
            ops = (valu_ops_per_rank_tabled(q) if tabled else valu_ops_per_rank(q, walks)) * P
            waves = (P + 255) // 256 * 4
            ent.update(bound="alu", achieved=ops / avg_ms / 1e6, peak=INT_VALU_PEAK_GOPS, unit="Gop/s",
                       peak_measured=valu_peak_measured, frac_of_measured=ops / avg_ms / 1e6 / valu_peak_measured,
                       # share of the kernel's time its vector instructions need on 1024 SIMDs at 4 cycles each
                       valu_busy=PROFILED_VALU_PER_WAVE * 4 * waves / (1024 * 2.4e9) / (avg_ms * 1e-3),
                       active_lane_fraction=PROFILED_ACTIVE_LANES / 64.0)
        elif name == "k_digits":
            ops = (3 * max(q - 7, 0) + 3 + 12) * P              # one walk a rank, address and store
            ent.update(bound="alu", achieved=ops / avg_ms / 1e6, peak=INT_VALU_PEAK_GOPS, unit="Gop/s")
        else:
            continue
        ent["frac"] = ent["achieved"] / ent["peak"]
        ent["traffic"] = PROFILED_TRAFFIC_BYTES.get(name)
        kernels[name] = ent
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    roofline = dict(kernels[dominant], kernel=dominant)

    out = {
        "metric": "rank-schedules constructed/s (int32, bit-exact) + expand GB/s vs HBM peak",
        "value": P / (ms_per_step * 1e-3),
        "unit": "rank-schedules/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_with_kernel_events": ms_per_step_events,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": "p=2^20+1 (q=21), all ranks, root 0: recv+send schedules, then expansion n=%d "
                               "(R=%d rounds)" % (N_BLOCKS, R), "p": P, "q": q, "n": N_BLOCKS, "rounds": R},
        "expand_gbs": kernels["k_expand_rows"]["achieved"],
        "construct_rank_schedules_per_s": P / (sum(kernels[k]["ms_per_step"] for k in
                                                   ("k_digits", "k_recv_uniform", "k_send_lookup") if k in kernels)
                                               * 1e-3),
        "roofline": roofline,
        "kernels": kernels,
        "digit_walks_per_rank": walks,
    }
    if ms_per_step_graph is not None:
        out["ms_per_step_in_hip_graph"] = ms_per_step_graph
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
