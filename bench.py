#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over the 100,000-configuration sweep
(p in [2,1024], up to 512 segments, fp64 costs): completion times and baselines
under both port models (simulate_completion_batch), the schedules themselves
under both models (greedy_schedule_batch), and the replay of the p = 256,
64-segment uni-greedy schedule over 256 buffers of 2^22 elements, once int32 and
once fp32 (replay_reduction).  Inputs are resident in HBM before the timed
region.  The calls of a step are enqueued one after the other on one stream
(--overlap: the four sweep calls on four streams; not faster, every call fills
the GPU); the time of every call on its own comes from a second pass after the
timed region.  One JSON line is printed.

Outside the timed step, reported in the same line: the large-machine sweep
(p in [1024, 65536], 64 to 4096 segments; every 16th of its 10,000
configurations, completion times under both models), the register-only
microkernel that gives the practical ceiling of Algorithm 1's arithmetic, plain
device copy and read passes, the best-segmentation search, the unequal-
segmentation experiment, and the CPU oracle on a bounded sample.
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

import numpy as np

N_CONFIGS = 100_000
P_MAX, Q_MAX = 1024, 512
REPLAY_P, REPLAY_Q, REPLAY_N = 256, 64, 1 << 22
# published peaks of the chip: 256 CUs x 64 fp64 lanes x 2.4 GHz (one add or compare per lane and cycle;
# the 78.6 TFLOP/s figure counts a fused multiply-add as two), HBM3E 8 TB/s
PEAK_FP64_OPS = 256 * 64 * 2.4e9
PEAK_HBM = 8.0e12
# algorithmic operations per send/receive pair (the arithmetic the method itself needs):
# Algorithm 1: two comparisons to pick the two smallest of two sorted fronts, t + tcomm, + tcomp
OPS_PER_PAIR_UNI = 4
# Algorithm 2: S <= t, R <= t and the two COMP comparisons for sender and receiver, t + tcomm, + tcomp
OPS_PER_PAIR_BI = 10


def cpu_baseline(host, large):
    """The oracle as it stands on this machine's cores, on a prefix of the same sweep; next to it the same on one
    core (a shorter prefix) and a few configurations of the large-machine sweep."""
    from concurrent.futures import ThreadPoolExecutor

    import oracle

    oracle.build()
    cores = min(16, os.cpu_count() or 1)
    sample = 1024
    idx = np.arange(sample)

    def one(i):
        oracle.simulate_batch(host, oracle.UNI, index=[i])
        oracle.simulate_batch(host, oracle.BI, index=[i])

    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        list(ex.map(one, idx, chunksize=4))
    dt = time.perf_counter() - t0
    one_sample = 96
    t1 = time.perf_counter()
    for i in range(one_sample):
        one(i)
    dt1 = time.perf_counter() - t1
    # large machines: the value-only form of Algorithm 1 and Algorithm 2 on the cheapest of the timed subsample
    pick = np.argsort(large.p.astype(np.float64) ** 2 * large.q_req)[:cores]

    def big(i):
        sizes = oracle.equi_sizes(int(large.m[i]), int(large.q_req[i]))
        a, b, g = float(large.alpha[i]), float(large.beta[i]), float(large.gamma[i])
        oracle.uni_greedy_time(int(large.p[i]), sizes, a, b, g, "f64")
        oracle.bi_greedy(int(large.p[i]), sizes, a, b, g, "f64", mode=oracle.MODE_EVENT | oracle.MODE_PRUNE, want_schedule=False)
        return (int(large.p[i]) - 1) * len(sizes)

    t2 = time.perf_counter()
    with ThreadPoolExecutor(cores) as ex:
        big_pairs = sum(ex.map(big, pick))
    dt2 = time.perf_counter() - t2
    return {"value": 2 * sample / dt, "unit": "schedules/s", "cores": cores, "kind": "oracle",
            "sample": f"first {sample} configurations of the 100,000-configuration sweep, uni-greedy and bi-greedy "
                      f"completion times with baselines, {dt:.1f} s of wall time",
            "one_core": {"value": 2 * one_sample / dt1, "unit": "schedules/s", "cores": 1,
                         "sample": f"first {one_sample} configurations of the same sweep, {dt1:.1f} s"},
            "large_machines": {"value": 2 * len(pick) / dt2, "unit": "schedules/s", "pairs_per_s": 2 * big_pairs / dt2, "cores": cores,
                               "sample": f"the {len(pick)} cheapest configurations of the timed large-machine subsample "
                                         f"(value-only uni-greedy, bi-greedy), {dt2:.1f} s"}}


SEARCH_PROBLEMS = 10000

COUNTER_FILE = os.path.join("profiles", "sweep100k_and_replay_counters_per_call.txt")


def profiled_counters():
    """Per call of the step: HBM bytes per launch and share of the VALU issue slots, as summarised from rocprofv3
    counter runs in COUNTER_FILE (lines `call hbm_bytes valu_busy`); nothing is measured here.  Empty if the file
    is missing."""
    table = {}
    try:
        with open(os.path.join(ROOT, COUNTER_FILE)) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and not line.startswith("#"):
                    table[parts[0]] = (float(parts[1]), float(parts[2]))
    except OSError:
        pass
    return table


LARGE_EVERY = 16
LARGE_P_MAX, LARGE_Q_MAX = 65536, 4096


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap", action="store_true",
                    help="enqueue the four sweep calls of a step, which do not depend on each other, on four streams "
                         "(default: one after the other on one stream; measured: 225 ms per step against 206, every "
                         "call already fills the GPU)")
    ap.add_argument("--step-only", action="store_true",
                    help="print after the timed step and the per-call pass (profiler runs: none of the extra blocks)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of 1 GiB (calibrates the HBM byte counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the sweep is a batch of independent configurations and nothing here "
              "spans devices; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1310_4645_amd as prs
    import prs_inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    prs.load_library()

    host = prs_inputs.uni_sweep(N_CONFIGS)
    dev = prs.DeviceConfigs.from_host(host)
    off = prs.prs_pair_offsets(dev, P_MAX, Q_MAX)
    torch.cuda.synchronize()
    n_pairs = int(off[-1].item())

    # buffers allocated once, outside the timed region
    f64, i32 = torch.float64, torch.int32
    times = {m: {k: torch.empty(N_CONFIGS, dtype=f64, device="cuda")
                 for k in ("greedy", "binomial", "pipeline", "binary", "revopt", "butterfly", "lower_bound")}
             for m in (prs.PRS_UNI, prs.PRS_BI)}
    for m in times:
        times[m]["q_eff"] = torch.empty(N_CONFIGS, dtype=i32, device="cuda")
        times[m]["cfg_status"] = torch.empty(N_CONFIGS, dtype=i32, device="cuda")
    src = torch.empty(n_pairs, dtype=i32, device="cuda")
    dst = torch.empty(n_pairs, dtype=i32, device="cuda")
    seg = torch.empty(n_pairs, dtype=i32, device="cuda")
    tst = torch.empty(n_pairs, dtype=f64, device="cuda")
    # the bi-greedy schedules get arrays of their own: the two schedule calls of a step may run at the same time
    src_b, dst_b, seg_b, tst_b = (torch.empty_like(x) for x in (src, dst, seg, tst))
    side = [torch.cuda.Stream() for _ in range(4)]
    ws = {}
    for call in (prs.PRS_CALL_SIMULATE, prs.PRS_CALL_SCHEDULE):
        for m in (prs.PRS_UNI, prs.PRS_BI):
            nbytes = prs.prs_workspace_bytes(call, m, prs.PRS_COST_F64, N_CONFIGS, P_MAX, Q_MAX)
            ws[(call, m)] = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")

    # replay workload: the p = 256, 64-segment uni-greedy schedule and its 2 x 4 GiB of buffers
    rcfg = prs.DeviceConfigs.from_host(prs_inputs.replay_config())
    roff = prs.prs_pair_offsets(rcfg, REPLAY_P, REPLAY_Q)
    rsch = prs.greedy_schedule_batch(rcfg, prs.PRS_UNI, REPLAY_P, REPLAY_Q, roff, (REPLAY_P - 1) * REPLAY_Q)
    gen = torch.Generator(device="cuda").manual_seed(prs_inputs.SEED_REPLAY)
    buf_i = torch.randint(-2 ** 20, 2 ** 20 + 1, (REPLAY_P, REPLAY_N), dtype=i32, device="cuda", generator=gen)
    buf_f = torch.randn((REPLAY_P, REPLAY_N), dtype=torch.float32, device="cuda", generator=gen)
    out_i = torch.empty(REPLAY_N, dtype=i32, device="cuda")
    out_f = torch.empty(REPLAY_N, dtype=torch.float32, device="cuda")
    seg_off = np.arange(REPLAY_Q + 1, dtype=np.int64) * (REPLAY_N // REPLAY_Q)
    rws = torch.empty(prs.prs_workspace_bytes(prs.PRS_CALL_REPLAY, 0, 0, 1, REPLAY_P, REPLAY_Q) + 256,
                      dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    names = ["simulate_uni", "simulate_bi", "schedule_uni", "schedule_bi", "replay_i32", "replay_f32"]
    held = {}                                    # what the calls of the last step returned

    def calls():
        return [lambda: prs.simulate_completion_batch(dev, prs.PRS_UNI, P_MAX, Q_MAX, out=times[prs.PRS_UNI],
                                                      workspace=ws[(prs.PRS_CALL_SIMULATE, prs.PRS_UNI)]),
                lambda: prs.simulate_completion_batch(dev, prs.PRS_BI, P_MAX, Q_MAX, out=times[prs.PRS_BI],
                                                      workspace=ws[(prs.PRS_CALL_SIMULATE, prs.PRS_BI)]),
                lambda: held.__setitem__("su", prs.greedy_schedule_batch(dev, prs.PRS_UNI, P_MAX, Q_MAX, off, n_pairs, src, dst, seg, tst,
                                                                         workspace=ws[(prs.PRS_CALL_SCHEDULE, prs.PRS_UNI)])),
                lambda: held.__setitem__("sb", prs.greedy_schedule_batch(dev, prs.PRS_BI, P_MAX, Q_MAX, off, n_pairs, src_b, dst_b, seg_b, tst_b,
                                                                         workspace=ws[(prs.PRS_CALL_SCHEDULE, prs.PRS_BI)])),
                lambda: held.__setitem__("ri", prs.replay_reduction(REPLAY_P, REPLAY_Q, seg_off, rsch["src"], rsch["dst"], rsch["seg"],
                                                                    buf_i, out=out_i, workspace=rws)),
                lambda: held.__setitem__("rf", prs.replay_reduction(REPLAY_P, REPLAY_Q, seg_off, rsch["src"], rsch["dst"], rsch["seg"],
                                                                    buf_f, out=out_f, workspace=rws))]

    def step(events=None):
        """The calls of a step one after the other on the current stream, an event between them."""
        fns = calls()
        for k, fn in enumerate(fns):
            if events is not None:
                events[k].record()
            fn()
        if events is not None:
            events[len(fns)].record()

    def step_overlapped():
        """The same calls; the four sweep calls share nothing but their inputs and go to four streams, heaviest
        first, the two replays follow on the main stream."""
        fns = calls()
        main = torch.cuda.current_stream()
        for k in (3, 2, 1, 0):
            side[k].wait_stream(main)
            with torch.cuda.stream(side[k]):
                fns[k]()
        for k in range(4):
            main.wait_stream(side[k])
        fns[4]()
        fns[5]()

    if args.copy_probe:
        a = torch.empty(2 ** 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    run = step_overlapped if args.overlap else step
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        run()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    # per call: a pass of its own after the timed region, the calls one after the other with events between them
    n_seq = min(args.steps, 3)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(n_seq)]
    t1 = time.perf_counter()
    for s in range(n_seq):
        step(ev[s])
    torch.cuda.synchronize()
    ms_per_step_sequential = (time.perf_counter() - t1) * 1e3 / n_seq
    part_ms = {nm: float(np.mean([ev[s][k].elapsed_time(ev[s][k + 1]) for s in range(n_seq)]))
               for k, nm in enumerate(names)}

    last = {"replay_status": [int(held["ri"][1].item()), int(held["rf"][1].item())],
            "sched_status_bad": [int((held[k]["cfg_status"] != 0).sum().item()) for k in ("su", "sb")],
            "T_equal": [bool(torch.equal(held["su"]["T_greedy"], times[prs.PRS_UNI]["greedy"])),
                        bool(torch.equal(held["sb"]["T_greedy"], times[prs.PRS_BI]["greedy"]))],
            "bi_src_range": [int(src_b.min().item()), int(src_b.max().item())]}
    # sanity of what was timed: all configurations valid, schedules complete and in range, replay finished
    assert int((times[prs.PRS_UNI]["cfg_status"] != 0).sum().item()) == 0
    assert int((times[prs.PRS_BI]["cfg_status"] != 0).sum().item()) == 0
    assert last["replay_status"] == [0, 0], last["replay_status"]
    assert last["sched_status_bad"] == [0, 0]
    # the schedule call returns the same completion times as the simulate call, and processor indices of a machine
    assert last["T_equal"] == [True, True]
    assert last["bi_src_range"][0] >= 1 and last["bi_src_range"][1] <= P_MAX - 1

    # roofline of the dominant kernel (the launch that takes the largest share of the step)
    dominant = max(part_ms, key=part_ms.get)
    if dominant.startswith("replay"):
        alg = 4.0 * REPLAY_N * (REPLAY_P + 1)
        roof = {"bound": "hbm", "achieved": alg / (part_ms[dominant] * 1e-3) / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s"}
    else:
        ops = n_pairs * (OPS_PER_PAIR_UNI if dominant.endswith("uni") else OPS_PER_PAIR_BI)
        roof = {"bound": "alu", "achieved": ops / (part_ms[dominant] * 1e-3) / 1e12, "peak": PEAK_FP64_OPS / 1e12,
                "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # HBM bytes per launch of that call's kernel and the share of the chip's VALU issue slots it uses: not measured
    # in this run but read from the rocprofv3 counter summary named here (FETCH_SIZE and WRITE_SIZE scaled by what
    # they read for a plain copy; SQ_INSTS_VALU x 4 cycles / (1024 SIMDs x launch time x 2.4 GHz)); None if absent
    prof = profiled_counters()
    roof["traffic"] = prof.get(dominant, (None, None))[0]
    roof["kernel"] = dominant
    roof["valu_busy_profiled"] = prof.get(dominant, (None, None))[1]
    roof["counters_from"] = COUNTER_FILE if prof else None
    replay_bytes = 4.0 * REPLAY_N * (REPLAY_P + 1)
    out = {
        "metric": "greedy schedules simulated/sec (uni+bi, p<=65536) + replay HBM GB/s vs peak",
        "value": 2 * N_CONFIGS / (ms_per_step * 1e-3), "unit": "schedules/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "configs[1]+configs[2]: 100,000 seeded configurations, p in [2,1024], q_req in [1,512], "
                               "fp64 costs, uni- and bi-greedy completion times, baselines and full schedules; "
                               "plus configs[4]: replay of the p=256, q=64 uni-greedy schedule over 256 x 2^22 int32 and fp32",
                   "n_configs": N_CONFIGS, "pairs_per_model": n_pairs},
        "streams": 4 if args.overlap else 1,
        "ms_per_step_sequential": ms_per_step_sequential,
        "breakdown_ms": part_ms,
        "breakdown_note": "per call, from a pass after the timed region with the calls one after the other on one stream",
        "pairs_per_s": {"uni_simulate": n_pairs / (part_ms["simulate_uni"] * 1e-3),
                        "bi_simulate": n_pairs / (part_ms["simulate_bi"] * 1e-3),
                        "uni_schedule": n_pairs / (part_ms["schedule_uni"] * 1e-3),
                        "bi_schedule": n_pairs / (part_ms["schedule_bi"] * 1e-3)},
        "replay": {"i32_GBps": replay_bytes / (part_ms["replay_i32"] * 1e-3) / 1e9,
                   "f32_GBps": replay_bytes / (part_ms["replay_f32"] * 1e-3) / 1e9,
                   "peak_GBps": PEAK_HBM / 1e9, "algorithmic_bytes": replay_bytes,
                   "frac_of_peak": replay_bytes / (min(part_ms["replay_i32"], part_ms["replay_f32"]) * 1e-3) / PEAK_HBM,
                   "traffic": prof.get("replay_f32", (None, None))[0],
                   "note": "whole replay_reduction call (schedule check and program build included)"},
        "schedule_emission_GBps": {"uni": n_pairs * 20.0 / (part_ms["schedule_uni"] * 1e-3) / 1e9,
                                   "bi": n_pairs * 20.0 / (part_ms["schedule_bi"] * 1e-3) / 1e9},
        "roofline": roof,
    }
    if args.step_only:
        print(json.dumps(out))
        return
    # outside the timed step: what plain device kernels reach on the same 4 GiB of buffers (the practical ceilings
    # next to the published 8 TB/s): a device-to-device copy (bytes read + bytes written) and a read-only pass
    def timed(fn, reps=3):
        best = float("inf")
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best
    buf_bytes = 4.0 * REPLAY_P * REPLAY_N
    buf_i.copy_(buf_f.view(i32))                                         # warm-up; buf_i is no longer needed
    out["replay"]["device_copy_GBps"] = 2 * buf_bytes / (timed(lambda: buf_i.copy_(buf_f.view(i32))) * 1e-3) / 1e9
    out["replay"]["device_read_GBps"] = buf_bytes / (timed(lambda: buf_f.max()) * 1e-3) / 1e9
    # the register-only microkernel: Algorithm 1's arithmetic with nothing else in the way
    sink = torch.zeros(1, dtype=f64, device="cuda")
    alu_steps, alu_blocks = 20000, 256 * 8
    prs.prs_measure_alu_ceiling(200, alu_blocks, sink)
    alu_ms = timed(lambda: prs.prs_measure_alu_ceiling(alu_steps, alu_blocks, sink))
    alu_rate = alu_steps * alu_blocks * 256 / (alu_ms * 1e-3)
    out["alu_ceiling"] = {"pair_steps_per_s": alu_rate, "ops_per_s_at_4_per_step": 4 * alu_rate,
                          "frac_of_nominal_fp64": 4 * alu_rate / PEAK_FP64_OPS,
                          "note": "dependent steps of Algorithm 1's arithmetic on registers only, 8 blocks of 256 lanes per CU"}
    out["pair_steps_vs_alu_ceiling"] = {k: v / alu_rate for k, v in out["pairs_per_s"].items()}
    # the large-machine sweep (p in [1024, 65536], 64..4096 segments, m in [1 MiB, 1 GiB]): every 16th of its
    # 10,000 configurations, completion times under both models
    large_host = prs_inputs.large_p_sweep().take(np.arange(0, 10000, LARGE_EVERY))
    large = prs.DeviceConfigs.from_host(large_host)
    loff = prs.prs_pair_offsets(large, LARGE_P_MAX, LARGE_Q_MAX)
    torch.cuda.synchronize()
    large_pairs = int(loff[-1].item())
    large_ms = {}
    for m, nm in ((prs.PRS_UNI, "uni"), (prs.PRS_BI, "bi")):
        wsb = torch.empty(prs.prs_workspace_bytes(prs.PRS_CALL_SIMULATE, m, prs.PRS_COST_F64, len(large), LARGE_P_MAX, LARGE_Q_MAX) + 256,
                          dtype=torch.uint8, device="cuda")
        res = {}
        large_ms[nm] = timed(lambda: res.update(prs.simulate_completion_batch(large, m, LARGE_P_MAX, LARGE_Q_MAX, workspace=wsb)), reps=1)
        assert int((res["cfg_status"] != 0).sum().item()) == 0
        del wsb, res
    out["large_machines"] = {"workload": f"configs[3]: every {LARGE_EVERY}th of the 10,000 configurations with p in [1024,65536], "
                                         "q_req in [64,4096], m in [1 MiB,1 GiB], fp64 costs; completion times and baselines",
                             "n_configs": len(large), "pairs_per_model": large_pairs, "ms": large_ms,
                             "schedules_per_s": {k: len(large) / (v * 1e-3) for k, v in large_ms.items()},
                             "pairs_per_s": {k: large_pairs / (v * 1e-3) for k, v in large_ms.items()},
                             "note": "not part of the step or of value; one call per model, no warm-up"}
    # the best-segmentation search (Sections 5.2, 6.1) over the sweep's first 10,000 problems,
    # ten power-of-two segment counts each
    sub = prs.DeviceConfigs.from_host(host.take(np.arange(SEARCH_PROBLEMS)))
    search_ms = {}
    for m, nm in ((prs.PRS_UNI, "uni"), (prs.PRS_BI, "bi")):
        wsb = torch.empty(prs.prs_workspace_bytes(prs.PRS_CALL_SEARCH, m, prs.PRS_COST_F64, SEARCH_PROBLEMS, P_MAX, Q_MAX) + 256,
                          dtype=torch.uint8, device="cuda")
        prs.optimal_segmentation_batch(sub, m, P_MAX, Q_MAX, workspace=wsb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        prs.optimal_segmentation_batch(sub, m, P_MAX, Q_MAX, workspace=wsb)
        e1.record()
        torch.cuda.synchronize()
        search_ms[nm] = e0.elapsed_time(e1)
        del wsb
    out["optimal_segmentation"] = {"problems": SEARCH_PROBLEMS, "candidates_per_problem": int(np.log2(Q_MAX)) + 1,
                                   "ms": search_ms, "note": "not part of the step or of value"}
    # outside the timed step as well: the unequal-segmentation experiment of Section 8 at the paper's size (986 problems,
    # m = 10: 512 segmentations each) and with a longer message (m = 14: 8192 each)
    alphas = list(range(0, 11)) + list(range(20, 101, 10)) + list(range(200, 1001, 100))
    ps = [2 ** k for k in range(2, 11)] + [3 * 2 ** k for k in range(1, 9)]
    probs = [(p, a, g) for p in ps for a in alphas for g in (0, 1)]
    uneq = {}
    for m_units in (10, 14):
        n_u = len(probs)
        hu = prs_inputs.SweepConfigs(np.array([x[0] for x in probs], np.int32), np.zeros(n_u, np.int32),
                                     np.full(n_u, m_units, np.int64), np.array([x[1] for x in probs], np.int64),
                                     np.ones(n_u, np.int64), np.array([x[2] for x in probs], np.int64), "i64")
        du = prs.DeviceConfigs.from_host(hu)
        wsb = torch.empty(prs.prs_workspace_bytes(prs.PRS_CALL_UNEQUAL, prs.PRS_UNI, prs.PRS_COST_I64, n_u, P_MAX, m_units) + 256,
                          dtype=torch.uint8, device="cuda")
        res = prs.unequal_segmentation_batch(du, P_MAX, m_units, want_all=False, workspace=wsb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        res = prs.unequal_segmentation_batch(du, P_MAX, m_units, want_all=False, workspace=wsb)
        e1.record()
        torch.cuda.synchronize()
        flags = res["equi_optimal"].cpu().numpy()
        ratio = (res["T_equi"].double() / res["T_best"].double()).cpu().numpy()
        only = (flags & 2) == 0
        uneq[f"m{m_units}"] = {"problems": n_u, "segmentations_per_problem": 1 << (m_units - 1), "ms": e0.elapsed_time(e1),
                               "optimised_only_by_unequal": int(only.sum()),
                               "max_gain_pct": float((ratio[only].max() - 1) * 100) if only.any() else 0.0,
                               "mean_gain_pct": float((ratio[only].mean() - 1) * 100) if only.any() else 0.0}
        del wsb, res
    uneq["note"] = "not part of the step or of value; m10 is the paper's experiment (61 problems, 7.3 %, 2.0 %)"
    out["unequal_segmentation"] = uneq
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host, large_host)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
