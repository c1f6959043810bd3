#!/usr/bin/env python3
"""Benchmark of the swap-executor hot path on one MI355X.

A step is one training iteration of a synthetic decoder with the whole hot path in it: trace
record per operator, sequence match, policy application, timeline scan, swap-out / release /
swap-in / wait around the operators, drain.  Activations are resident in HBM when the timed
region starts.

Without --config the headline workload is configuration 3 (7B-shape decoder, 97 GiB of activations
under a 48 GB budget, 56.5 GB swapped each way per step): --steps steps are timed after --warmup
warm-up steps, and the other configurations (1, 2, 5 executed, 4 planned at full size), a generated
policy under a memory limit, the stage loop of Algo. 1 and the profiler-hook overhead table are
measured with small fixed step counts and attached as `sub_records`.  With --config N only that
configuration is measured.

Prints ONE JSON line.  `value` is D2H + H2D bytes over the step's wall time; the fractions of the
host-link peak are given per direction against that direction's peak, measured in the same run
with pinned hipMemcpy (`pct_of_link_peak`).  `roofline` names the mover of the dominant direction
(copy kernel or copy engine) with its GB/s from HIP events, `cpu_baseline` is the CPU oracle timed
on this machine's host cores.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

# Every stream of the process beyond HIP's hardware queues (4 by default) shares a queue with another stream
# and stands still while that one's work runs; when it is the compute stream that a swap stream shares with,
# a step of configuration 2 takes 211-239 ms instead of 119 ms.  The library uses up to three streams of its own
# (swap-out, swap-in, the ring transfers; the trace kernels run on the swap-in stream) beside the compute
# stream, and this process keeps a few more alive (PyTorch's pooled side streams of the measurement modes), so
# the limit is raised to 32, above any count of live streams reached here.
os.environ["GPU_MAX_HW_QUEUES"] = str(max(32, int(os.environ.get("GPU_MAX_HW_QUEUES") or 0)))

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
# Memory traffic of one pack launch over its algorithmic bytes (read from HBM + written to the host),
# from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs scaled by a plain copy of known size
# (profiles/ss_copy_kernel_config2_hbm_traffic.md); a constant carried over from that profile, not a
# counter of this run.
PACK_TRAFFIC_RATIO = 1.011
PACK_TRAFFIC_SOURCE = "profiles/ss_copy_kernel_config2_hbm_traffic.md"

METRIC = "swap GB/s (D2H+H2D) as % of host-link peak; step-time overhead vs no-swap"
WORKLOADS = {
    1: "config 1: toy 2-layer block, layer-0 activations swapped",
    2: "config 2: 1.3B-shape decoder (hidden 2048, 24 layers, seq 2048, mb 1, bf16), "
       "activations of every other layer swapped, synthetic bf16 GEMMs on the compute stream",
    3: "config 3: 7B-shape decoder (hidden 4096, 32 layers, seq 4096, mb 1, bf16), 97 GiB of activations "
       "under a 48 GB budget, longest-idle-first policy, synthetic bf16 GEMMs on the compute stream",
    5: "config 5: 20,000 tensors of 4 KiB..4 MiB at random places of a 64 GB arena, two random orders, "
       "no compute stream work"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ---- CPU oracle legs ---------------------------------------------------------------------------------

def _threaded_round_trip(oracle, arena, staging, ap, threads):
    """the oracle's per-descriptor byte copies (swap_out of every descriptor, then swap_in of every
    descriptor) with the descriptor lists dealt round-robin to `threads` threads; returns seconds"""
    from concurrent.futures import ThreadPoolExecutor
    outs = [ap["descs_out"][i::threads] for i in range(threads)]
    ins = [ap["descs_in"][i::threads] for i in range(threads)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        t0 = time.perf_counter()
        list(ex.map(lambda d: oracle.swap_out(arena, staging, d), outs))
        list(ex.map(lambda d: oracle.swap_in(arena, staging, d), ins))
        return time.perf_counter() - t0


def cpu_baseline(cfgno, bpo, budget_s=6.0):
    """The oracle as it stands on the host cores, one step of the same workload: trace record, match,
    apply, scan on one thread; the byte round trip on one thread (in schedule order) and once more with
    min(16, cores) threads.  Configurations 1, 2, 5 in full; 3 and 4 on a 1/8 layer subset (4 of 32
    layers, budget 6 GB), which moves 1/8 of the bytes at the same tensor sizes."""
    import numpy as np
    import oracle
    import workloads as W
    from workloads import transformer as T
    from workloads.arena import place_tensors
    cores = len(os.sched_getaffinity(0))
    threads = max(1, min(16, cores))
    subset = ""
    if cfgno == 5:
        tr, pol, arena_bytes = W.build_small_tensor_stress()
        tr_cur = tr
    elif cfgno in (3, 4):
        shape = dataclasses.replace(T.config_shape(cfgno), layers=4)
        subset = " on a 1/8 layer subset (4 of 32 layers, budget 6 GB; bytes per step are 1/8 of the full configuration's)"
        tr = T.build_trace(shape)
        rows, _ = oracle.greedy_policy(tr.tensors, tr.events, tr.n_ops, 0, 6 * 10**9, bpo, min_bytes=1 << 20)
        pol = np.zeros(len(rows), dtype=W.POLICY_DT)
        for i, r in enumerate(rows):
            pol[i] = r
        tr_cur = tr if cfgno == 3 else T.build_trace(shape, iteration=1, perturb=dict(p_drop=0.1, p_insert=0.1,
                                                                                     moe_max=8, seq_jitter=0.15))
        arena_bytes = None
    else:
        tr = T.build_trace(T.config_shape(cfgno))
        pol = T.config_swap_set(tr, cfgno)
        tr_cur, arena_bytes = tr, None
    anchors = [(int(p["ref_op"]), int(p["out_slot"])) for p in pol]
    ref_ops, _ = oracle.record_trace(oracle.TraceRecorder(), tr)
    ref_t = oracle.ops_tuples(ref_ops)

    def trace_work():
        rec = oracle.TraceRecorder()
        if tr_cur is not tr:
            oracle.record_trace(rec, tr)            # same interning order as the reference iteration
        t = [time.perf_counter()]
        ops, ev = oracle.record_trace(rec, tr_cur)                                     # a1
        t.append(time.perf_counter())
        m = oracle.match_sequence(ref_t, oracle.ops_tuples(ops), anchors)              # a3
        t.append(time.perf_counter())
        ap = oracle.apply_policy(pol, m["new_idx"], tr_cur.tensors, bpo)               # a4
        t.append(time.perf_counter())
        oracle.timeline_scan(ev, ap["policy_events"], tr_cur.n_ops, 0, 1 << 62)        # a2
        t.append(time.perf_counter())
        return ap, [t[i + 1] - t[i] for i in range(4)], len(ev)
    ap, dt, n_ev = trace_work()
    swapped = {r[2]: (r[5], r[6]) for r in ap["resolved"] if not r[3] & 3}
    if arena_bytes is None:
        arena_bytes = place_tensors(tr_cur.tensors, swapped=swapped)
        ap, dt, n_ev = trace_work()                  # descriptors with the placed offsets
    arena = np.zeros(arena_bytes, dtype=np.uint8)        # pages are committed when first written
    staging = np.zeros(max(1, ap["staging_bytes"]), dtype=np.uint8)
    oracle.execute_schedule(arena, staging, ap)          # warm-up: commits the pages that are touched
    reps, legs, t_bytes = 0, [0.0] * 4, 0.0
    while reps < 10 and (reps == 0 or sum(legs) + t_bytes < budget_s):  # bounded: at most ten steps or budget_s seconds
        if reps:
            ap, dt, n_ev = trace_work()
        reps += 1
        t1 = time.perf_counter()
        oracle.execute_schedule(arena, staging, ap)                                    # a5-a7 (bytes)
        t_bytes += time.perf_counter() - t1
        legs = [a + b for a, b in zip(legs, dt)]
    legs = [x / reps for x in legs]
    t_bytes /= reps
    t_trace = sum(legs)
    moved = 2 * sum(d[2] for d in ap["descs_out"])
    t_thr = _threaded_round_trip(oracle, arena, staging, ap, threads) if moved else 0.0
    n_ops = tr_cur.n_ops
    return {"value": round(moved / (t_trace + t_bytes) / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%d step(s) of configuration %d%s, %.3f GB each way per step; mean per step on one thread: "
                      "record+match+apply+scan %.4f s, byte round trip %.4f s; host has %d cores available"
                      % (reps, cfgno, subset, moved / 2e9, t_trace, t_bytes, cores),
            "byte_round_trip_gbps_1_thread": round(moved / t_bytes / 1e9, 3) if t_bytes > 0 else None,
            "byte_round_trip_gbps_threads": round(moved / t_thr / 1e9, 3) if t_thr > 0 else None,
            "threads": threads,
            "trace_work_us_1_thread": {"record": round(legs[0] * 1e6, 1), "match": round(legs[1] * 1e6, 1),
                                       "apply": round(legs[2] * 1e6, 1), "scan": round(legs[3] * 1e6, 1)},
            "record_ops_per_s": round(n_ops / legs[0]) if legs[0] > 0 else None,
            "scan_events_per_s": round((n_ev + len(ap["policy_events"])) / legs[3]) if legs[3] > 0 else None,
            "operators": n_ops, "events": n_ev, "anchors": len(anchors)}


def cpu_baseline_safe(cfgno, bpo, budget_s=6.0):
    try:
        return cpu_baseline(cfgno, bpo, budget_s)
    except Exception as e:                              # the GPU figures stand on their own
        return {"value": None, "unit": "GB/s", "cores": 1, "kind": "oracle",
                "sample": "failed: %s: %s" % (type(e).__name__, e)}


# ---- modes that print a line of their own -------------------------------------------------------------

def run_swap_only(B, torch, args, path, path_in):
    from workloads.harness import SwapRun
    run = SwapRun(B, torch, args.config or 2, swap=True, bpo=args.bpo if args.bpo > 0 else 10 << 20,
                  bpo_in=4 << 20, copy_path=path, copy_path_in=path_in, copy_workgroups=args.workgroups,
                  flags=B.SS_CFG_TIMING | B.SS_CFG_KEEP_LATE, compute=False)
    for _ in range(args.warmup + args.steps):
        run.step()
        log("swap-only step done")
    torch.cuda.synchronize()
    out_ms = [x for x in B.ss_batch_ms_all(run.ctx, 0).tolist() if x >= 0]
    nob = run.last["applied"]["n_out_batches"]
    line = {"mode": "swap-only", "bytes_each_way": run.bytes_each_way, "out_batches": int(nob),
            "in_batches": int(run.last["applied"]["n_in_batches"]),
            "avg_pack_launch_ms": round(sum(out_ms) / len(out_ms), 4),
            "bytes_per_pack_launch": run.bytes_each_way // nob}
    run.close()
    return line


def record_config4(B, torch, np, iterations=20, cpu=True):
    """varying sequences at full 7B size: what is measured is the per-iteration trace work (record is part
    of the step itself; here: match or align, apply, scan, top-up) and where the anchors land; bytes are
    not moved here (the larger iterations need more pinned staging than a host may give; execution at 7B
    tensor sizes is covered by the GPU tests)"""
    from workloads.harness import VaryingRun
    from workloads import transformer as T
    shape = T.config_shape(4)
    pert = dict(p_drop=0.1, p_insert=0.1, moe_max=8, seq_jitter=0.15)
    out, summary = {}, {}
    for name, mf in (("keyed_ordinals", 0), ("aligned", B.SS_MATCH_ALIGN)):
        run = VaryingRun(B, torch, shape, 48 * 10**9, 256 << 20, min_bytes=1 << 20, perturb=pert, compute=False,
                         match_flags=mf)
        tr0 = T.build_trace(shape)
        rows = []
        for it in range(iterations):
            p = run.plan(it)
            tr = p["trace"]
            truth = {b: j for j, b in enumerate(tr.op_base) if b is not None}
            want = np.array([truth.get(tr0.op_base[i], -1) for i in run.anchors["ref_op"].tolist()])
            got = p["match"]["new_idx"]
            rows.append(dict(it=it, ops=tr.n_ops, seq=tr.seq, similar=bool(p["match"]["similar"]),
                             stage=int(p["match"]["stage"]), anchors=len(got),
                             landed_on_true_operator=int((got == want).sum()),
                             landed_elsewhere=int(((got != want) & (got >= 0)).sum()),
                             unmatched=int((got < 0).sum()), carried=len(p["carried"]), topped_up=int(p["topped"]),
                             peak_gb=round(p["scan"]["peak"] / 1e9, 2),
                             host_ms={k: round(v, 3) for k, v in p["host_ms"].items()}))
        run.close()
        out[name] = rows
        later = rows[1:]
        n_anchor = sum(r["anchors"] for r in later)
        summary[name] = {
            "anchors_on_true_operator_or_correctly_gone_pct": round(
                100 * sum(r["landed_on_true_operator"] for r in later) / max(1, n_anchor), 1),
            "anchors_elsewhere_pct": round(100 * sum(r["landed_elsewhere"] for r in later) / max(1, n_anchor), 1),
            "items_topped_up": sum(r["topped_up"] for r in later),
            "max_peak_gb": max(r["peak_gb"] for r in later),
            "host_ms_per_iteration": {k: round(sum(r["host_ms"][k] for r in later) / len(later), 3)
                                      for k in later[0]["host_ms"]}}
        log("config 4 planning, %s: %s" % (name, summary[name]))
    work = [sum(r["host_ms"].values()) for r in out["aligned"][1:]]
    rec = {"metric": "trace work per iteration (match or align, apply, scan, top-up), host wall ms",
           "value": round(sum(work) / len(work), 3), "unit": "ms", "n_gpus": 1, "steps": iterations - 1, "warmup": 1,
           "ms_per_step": round(sum(work) / len(work), 3), "higher_is_better": False, "scaling": "weak",
           "vs_baseline": None, "dtype": "u8", "data": "synthetic",
           "config": {"workload": "config 4: 7B-shape decoder, operator sequence perturbed every iteration (drop / "
                                  "insert 0.1, 0-8 branch operators per layer, sequence length +-15 %), policy of "
                                  "iteration 0 re-anchored online under a 48 GB budget; planning only"},
           "summary": summary, "iterations": out}
    if cpu:
        rec["cpu_baseline"] = cpu_baseline_safe(4, 256 << 20)
    return rec


def record_staged(B, torch, bw, cfgno, limit_frac, steps):
    from workloads.harness import StagedRun
    from workloads import transformer as T
    shape = T.config_shape(cfgno)
    tr0 = T.build_trace(shape)
    link = min(bw["d2h_gbps"], bw["h2d_gbps"]) * 1e9
    run = StagedRun(B, torch, lambda it: tr0, limit_frac=limit_frac, link_bytes_per_s=link,
                    g_fwd=shape.layers, g_bwd=shape.layers, min_bytes=1 << 16, flags=B.SS_CFG_TIMING)
    lg = []
    for it in range(9 + steps):
        e = run.iteration(it)
        e.pop("result")
        lg.append(e)
        log("iteration %d stage %d: %.1f ms, %d tensors, %.0f MB each way" %
            (it, e["stage"], e["ms"], e["n_items"], e["bytes"] / 1e6))
    run.close()
    stable = [e for e in lg if e["stage"] == 2]
    warm = [e for e in lg if e["stage"] == 0][1:]
    t_stable = sum(e["ms"] for e in stable) / len(stable) * 1e-3
    t_warm = sum(e["ms"] for e in warm) / len(warm) * 1e-3
    return {
        "metric": METRIC, "value": round(2 * stable[0]["bytes"] / t_stable / 1e9, 3), "unit": "GB/s", "n_gpus": 1,
        "steps": len(stable), "warmup": 9, "ms_per_step": round(t_stable * 1e3, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config %d trace under the stage loop of Algo. 1 (m = 2, n = 5): WarmUp without "
                               "swapping, GenPolicy with one generated policy per iteration, Stable with the "
                               "fastest; memory limit %.2f x the no-swap peak" % (cfgno, limit_frac),
                   "policy_mode": "staged", "chosen_candidate": stable[0]["candidate"],
                   "bytes_each_way": stable[0]["bytes"], "tensors_swapped": stable[0]["n_items"],
                   "peak_bytes_with_policy": stable[0]["peak"]},
        "step_time": {"warmup_noswap_ms": round(t_warm * 1e3, 3), "stable_ms": round(t_stable * 1e3, 3),
                      "overhead_vs_noswap_pct": round(100 * (t_stable / t_warm - 1), 1)},
        "iterations": [{k: (round(v, 3) if isinstance(v, float) else v) for k, v in e.items()} for e in lg],
        "link_peak_measured": {k: round(v, 2) for k, v in bw.items()}}


def record_path_table(B, torch, np, bw):
    from workloads.layouts import DESC_DT
    from workloads.rng import SplitMix64
    arena_bytes = 8 << 30
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    rows = []
    for size in (4 << 10, 64 << 10, 1 << 20, 16 << 20, 256 << 20):
        n = max(4, min(20000, (1 << 30) // size))
        rng = SplitMix64(size, 3)
        slots = arena_bytes // size
        picks = sorted(set(rng.randint(slots) for _ in range(2 * n)))[:n]       # scattered, disjoint
        rng2 = SplitMix64(size, 4)
        order = sorted(range(len(picks)), key=lambda i: rng2.randint(1 << 30))  # shuffled issue order
        d = np.zeros(len(picks), dtype=DESC_DT)
        for k, i in enumerate(order):
            d[k] = (picks[i] * size, k * size, size, k, 0)
        start = np.array([0, len(d)], dtype=np.uint32)
        row = {"tensor_bytes": size, "tensors": len(d), "batch_bytes": int(size * len(d))}
        for pname, pcode, lookup in (("kernel", B.SS_PATH_KERNEL, 0), ("kernel_lds_lookup", B.SS_PATH_KERNEL, 1),
                                     ("engine", B.SS_PATH_ENGINE, 0)):
            cfg = B.ss_config_default()
            cfg.staging_bytes = int(size * len(d))
            cfg.copy_path = cfg.copy_path_in = pcode
            cfg.copy_desc_lookup = lookup
            cfg.flags = B.SS_CFG_TIMING
            ctx = B.ss_create(cfg)
            B.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
            B.ss_load_schedule(ctx, d, start, d, start)
            out_ms, in_ms = [], []
            for rep in range(4):
                B.ss_swap_out(ctx, 0)
                B.ss_swap_in(ctx, 0)
                B.ss_sync(ctx, B.SS_SYNC_DRAIN)
                if rep:
                    out_ms.append(B.ss_batch_ms(ctx, 0, 0)[0])
                    in_ms.append(B.ss_batch_ms(ctx, 1, 0)[0])
            B.ss_destroy(ctx)
            row[pname + "_d2h_gbps"] = round(row["batch_bytes"] / (min(out_ms) * 1e-3) / 1e9, 2)
            row[pname + "_h2d_gbps"] = round(row["batch_bytes"] / (min(in_ms) * 1e-3) / 1e9, 2)
        rows.append(row)
        log(row)
    return {"mode": "path-table", "link_peak_measured": {k: round(v, 2) for k, v in bw.items()},
            "columns": "kernel: ss_copy_kernel with the per-chunk descriptor table (the default); kernel_lds_lookup: the "
                       "same kernel with the batch's chunk-prefix table staged in LDS and searched per chunk; engine: one "
                       "hipMemcpyAsync per tensor; best of three repetitions of one 1 GiB batch, GB/s",
            "rows": rows}


def record_mover_table(B, torch, np, bw, args):
    """configuration 2 with every mover per direction inside the running step (copy kernel, copy engine, the
    rings), and what each mover costs a compute stream that does not wait for it: the backward pass of the
    no-swap step timed alone, beside copy-engine transfers, beside copy-kernel launches that saturate the
    link, and with as many marker / wait pairs on the compute stream as the schedule has swap-in batches"""
    from workloads.harness import SwapRun
    rows = []
    combos = [("kernel", "engine", {}), ("kernel", "kernel", {}), ("kernel", "kernel", dict(workgroups=16)),
              ("kernel", "kernel", dict(copy_cus=8)), ("kernel", "kernel", dict(copy_cus=16)),
              ("kernel", "kernel", dict(copy_cus=64)),
              ("engine", "engine", {}), ("engine", "kernel", {}), ("staged", "engine", {}), ("staged", "staged", {}),
              ("staged", "staged", dict(bare_ring=1))]
    # the whole table runs on a compute stream of its own: swap streams with a compute-unit mask synchronise with
    # the null stream (the runtime has no non-blocking form of them)
    own = torch.cuda.Stream()
    # the side stream of the last part is made and used now, before any context of the library exists: where a
    # stream lands among the hardware queues decides what a wait between two of them costs (40 us or 0.9 ms per
    # round trip were measured for the same loop)
    side = torch.cuda.Stream()
    for st_ in (own, side):
        with torch.cuda.stream(st_):
            torch.zeros(1, device="cuda")
    torch.cuda.synchronize()
    torch.cuda.set_stream(own)
    for p_out, p_in, kw in combos:
        o = argparse.Namespace(**vars(args))
        o.config, o.path, o.path_in, o.calibrate, o.no_cpu_baseline, o.no_stall_timing = 2, p_out, p_in, 0, True, True
        o.bpo = args.bpo if args.bpo > 0 else 11500000
        o.steps, o.warmup = min(args.steps, 8), max(args.warmup, 11)      # the stage machine needs nine iterations to settle
        o.copy_cus, o.bare_ring = 0, 0
        for k, v in kw.items():
            setattr(o, k, v)
        r = measure(B, torch, np, bw, o)
        rows.append({"swap_out": p_out, "swap_in": p_in, **kw, "ms_per_step": r["ms_per_step"],
                     "overhead_vs_floor_out_then_in_pct": r["step_time"]["overhead_vs_floor_out_then_in_pct"],
                     "d2h_pct_of_peak_while_copying": r["pct_of_link_peak"]["d2h_while_copying"],
                     "h2d_pct_of_peak_while_copying": r["pct_of_link_peak"]["h2d_while_copying"],
                     "d2h_pct_first_start_to_last_end": r["pct_of_link_peak"]["d2h_first_start_to_last_end"],
                     "h2d_pct_first_start_to_last_end": r["pct_of_link_peak"]["h2d_first_start_to_last_end"]})
        log("mover table: %s" % rows[-1])
    # what a mover costs a compute stream that never waits for it
    base = SwapRun(B, torch, 2, swap=False)
    n = base.tr.n_ops
    fb = list(base.tr.op_phase).index(1)
    nbytes = 256 << 20
    host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    dev = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    n_bg = 11                                      # background transfers of 256 MiB: about 50 ms of link traffic

    def kernel_ctx():
        from workloads.layouts import DESC_DT
        cfg = B.ss_config_default()
        cfg.staging_bytes = n_bg * nbytes
        cfg.copy_path = cfg.copy_path_in = B.SS_PATH_KERNEL
        c = B.ss_create(cfg)
        B.ss_bind(c, dev.data_ptr(), nbytes, side.cuda_stream)       # its swap streams order after `side`, which stays empty
        d = np.zeros(n_bg, dtype=DESC_DT)
        for b in range(n_bg):
            d[b] = (0, b * nbytes, nbytes, b, 0)
        start = np.arange(n_bg + 1, dtype=np.uint32)
        B.ss_load_schedule(c, d, start, d, start, np.arange(n_bg, dtype=np.uint32))
        return c
    kctx = kernel_ctx()

    def backward_ms(mode, pairs=0):
        cur = torch.cuda.current_stream()
        e1, e2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        every = max(1, (n - fb) // pairs) if pairs else 0
        if mode == "kernel_h2d":                   # the staging slots are filled first, outside the measurement
            for b in range(n_bg):
                B.ss_swap_out(kctx, b)
            torch.cuda.synchronize()
        for i in range(n):
            if i == fb:
                e1.record()
                if mode == "engine_h2d":
                    with torch.cuda.stream(side):
                        for _ in range(n_bg):
                            dev.copy_(host, non_blocking=True)
                elif mode == "kernel_h2d":
                    for b in range(n_bg):
                        B.ss_swap_in(kctx, b)
            if pairs and i >= fb and (i - fb) % every == 0:
                m = torch.cuda.Event(); m.record(cur)
                side.wait_event(m)
                d = torch.cuda.Event(); d.record(side)
                cur.wait_event(d)
            base.compute.run_op(i)
        e2.record()
        torch.cuda.synchronize()
        if mode == "kernel_h2d":
            B.ss_sync(kctx, B.SS_SYNC_DRAIN)
        return e1.elapsed_time(e2)
    costs = {}
    for label, mode, pairs in (("alone", None, 0), ("beside copy-engine transfers host to device", "engine_h2d", 0),
                               ("beside ss_copy_kernel launches host to device (64 workgroups)", "kernel_h2d", 0),
                               ("with 145 marker / wait pairs on the compute stream", None, 145)):
        for _ in range(3):
            backward_ms(mode, pairs)
        costs[label] = round(float(np.median([backward_ms(mode, pairs) for _ in range(5)])), 2)
        log("mover table: backward pass %s: %.2f ms" % (label, costs[label]))
    B.ss_destroy(kctx)
    torch.cuda.set_stream(torch.cuda.default_stream())
    base.close()
    return {"mode": "mover-table", "workload": WORKLOADS[2], "link_peak_measured": {k: round(v, 2) for k, v in bw.items()},
            "rows": rows, "noswap_backward_pass_ms": costs}


def record_transfer_cost_table(B, torch, np):
    """What 2.6-2.8 GB of host-to-device (and device-to-host) traffic costs a compute stream that nothing orders
    against it: the backward pass of configuration 2 without swapping, timed with HIP events, beside copy-engine
    transfers with and without another command on their stream, and beside the library's swap-ins by copy engine and by
    copy kernel, in few large and in many small batches."""
    from workloads.harness import SwapRun
    from workloads.layouts import DESC_DT
    side = torch.cuda.Stream()          # made first: where a stream lands among the hardware queues matters
    with torch.cuda.stream(side):
        torch.zeros(1, device="cuda")
    torch.cuda.synchronize()
    base = SwapRun(B, torch, 2, swap=False)
    n = base.tr.n_ops
    fb = list(base.tr.op_phase).index(1)
    M = 1 << 20
    host = torch.empty(2816 * M, dtype=torch.uint8, pin_memory=True)
    dev = torch.empty(2816 * M, dtype=torch.uint8, device="cuda")

    def backward_ms(traffic):
        e1, e2 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(n):
            if i == fb:
                e1.record()
                if traffic is not None:
                    traffic()
            base.compute.run_op(i)
        e2.record()
        torch.cuda.synchronize()
        return e1.elapsed_time(e2)

    def best(traffic, after=None):
        out = []
        for _ in range(4):
            out.append(backward_ms(traffic))
            if after is not None:
                after()
        return round(min(out[1:]), 2)

    flag_host = {nb: torch.zeros(nb, dtype=torch.uint8, pin_memory=True) for nb in (8, 65536)}
    flag_dev = {nb: torch.zeros(nb, dtype=torch.uint8, device="cuda") for nb in (8, 65536)}

    def transfer(k, d2h):
        a, b = host[k * 256 * M:(k + 1) * 256 * M], dev[k * 256 * M:(k + 1) * 256 * M]
        (a.copy_(b, non_blocking=True) if d2h else b.copy_(a, non_blocking=True))

    def plain(d2h, extra):
        def go():
            with torch.cuda.stream(side):
                for k in range(11):
                    transfer(k, (k % 2 == 0) if d2h == "mixed" else d2h)
                    if extra == "event" or (extra == "event_first" and k == 0) or (extra == "event_last" and k == 10):
                        torch.cuda.Event().record(side)
                    elif extra == "kernel":
                        dev[:64].zero_()
                    elif extra in ("flag8", "flag64k"):       # a second, small transfer behind each: a sequence number
                        nb = 8 if extra == "flag8" else 65536
                        flag_dev[nb].copy_(flag_host[nb], non_blocking=True)
        return go

    def threaded(d2h):
        """the transfers issued by a second host thread that waits for their stream after each"""
        import threading
        box = {}

        def work():
            with torch.cuda.stream(side):
                for k in range(11):
                    transfer(k, d2h)
                    side.synchronize()

        def go():
            box["t"] = threading.Thread(target=work)
            box["t"].start()

        def join():
            box["t"].join()
        return go, join
    rows = [{"traffic": "none", "backward_pass_ms": best(None)}]
    for d2h in (False, True):
        for extra, what in ((None, "nothing else on their stream"), ("event", "an event recorded on their stream after each"),
                            ("event_last", "one event recorded after the last of them"),
                            ("event_first", "one event recorded after the first of them"),
                            ("kernel", "a one-block kernel on their stream after each")):
            if d2h and extra in ("event_last", "event_first"):
                continue
            rows.append({"traffic": "11 copy-engine transfers of 256 MiB %s (PyTorch copy_), %s" % (
                "device to host" if d2h else "host to device", what), "backward_pass_ms": best(plain(d2h, extra))})
            log("transfer cost table: %s" % rows[-1])
    # what signalling completion through memory costs instead: a small transfer of a sequence number behind each
    # transfer, both directions on one stream, the transfers issued by a thread that waits for each on the host
    for d2h, extra, what in ((False, "flag64k", "host to device, each followed by a host-to-device transfer of 64 KiB"),
                             (False, "flag8", "host to device, each followed by a host-to-device transfer of 8 bytes"),
                             (True, "flag64k", "device to host, each followed by a host-to-device transfer of 64 KiB"),
                             ("mixed", None, "alternately device to host and host to device on one stream, nothing else on it")):
        rows.append({"traffic": "11 copy-engine transfers of 256 MiB %s" % what, "backward_pass_ms": best(plain(d2h, extra))})
        log("transfer cost table: %s" % rows[-1])
    for d2h in (False, True):
        go_, join_ = threaded(d2h)
        rows.append({"traffic": "11 copy-engine transfers of 256 MiB %s, issued by a second host thread that waits for "
                                "their stream after each" % ("device to host" if d2h else "host to device"),
                     "backward_pass_ms": best(go_, join_)})
        log("transfer cost table: %s" % rows[-1])
    del host
    for path, pname in ((B.SS_PATH_ENGINE, "copy engine"), (B.SS_PATH_KERNEL, "ss_copy_kernel")):
        for nb in (11, 33, 132):
            nbytes = (2640 // nb) * M
            cfg = B.ss_config_default()
            cfg.staging_bytes = nb * nbytes
            cfg.copy_path = B.SS_PATH_KERNEL
            cfg.copy_path_in = path
            c = B.ss_create(cfg)
            try:
                B.ss_bind(c, dev.data_ptr(), nb * nbytes, side.cuda_stream)      # ordered after `side`, which stays empty
                d = np.zeros(nb, dtype=DESC_DT)
                for b in range(nb):
                    d[b] = (b * nbytes, b * nbytes, nbytes, b, 0)
                st = np.arange(nb + 1, dtype=np.uint32)
                B.ss_load_schedule(c, d, st, d, st, np.arange(nb, dtype=np.uint32))

                def fill():
                    for b in range(nb):
                        B.ss_swap_out(c, b)
                    torch.cuda.synchronize()

                def go():
                    for b in range(nb):
                        B.ss_swap_in(c, b)

                def after():
                    B.ss_sync(c, B.SS_SYNC_DRAIN)
                    fill()
                fill()
                ms = best(go, after)
                B.ss_sync(c, B.SS_SYNC_DRAIN)
                rows.append({"traffic": "the library's swap-ins by %s, %d batches of %d MiB (a marker wait before, a done-event after each)"
                                        % (pname, nb, nbytes // M), "backward_pass_ms": ms})
                log("transfer cost table: %s" % rows[-1])
            finally:
                B.ss_destroy(c)
    base.close()
    return {"mode": "transfer-cost-table",
            "workload": "backward pass of configuration 2 without swapping (350 operators) beside 2.6-2.8 GB of traffic that "
                        "nothing orders against it; HIP events on the compute stream, best of three", "rows": rows}


def record_reuse_interval(B, torch, np, bw, cfgno, path, path_in):
    from paper_2509_11076_amd.executor import run_iteration_dispatch
    from workloads.harness import SwapRun
    link = min(bw["d2h_gbps"], bw["h2d_gbps"]) * 1e9
    base = SwapRun(B, torch, cfgno, swap=False)
    for _ in range(3):
        base.step_noswap()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        base.step_noswap()
    torch.cuda.synchronize()
    t_ns = (time.perf_counter() - t0) / 5
    n_ops = base.tr.n_ops
    base.close()
    del base
    torch.cuda.empty_cache()
    run = SwapRun(B, torch, cfgno, swap=True, bpo=max(1, int(link * 2 * t_ns / n_ops)),
                  bpo_in=max(1, int(link * t_ns / n_ops)), copy_path=path, copy_path_in=path_in,
                  flags=B.SS_CFG_TIMING | B.SS_CFG_KEEP_LATE)
    for _ in range(3):
        run.step()
    torch.cuda.synchronize()
    plan = run.plan()
    acts = plan["applied"]["actions"]
    issue_op, free_op = {}, {}
    for op, kind, tid, batch in acts.tolist():
        if kind == B.SS_ACT_OUT:
            issue_op.setdefault(batch, op)
        elif kind == B.SS_ACT_FREE:
            free_op[batch] = max(free_op.get(batch, 0), op)
    B.ss_trace_begin(run.ctx)
    seen_done, pending, n_query, t_query = {}, [], 0, 0.0

    def run_op(i):
        nonlocal n_query, t_query
        run.record(i)
        run.compute.run_op(i)
        # what a host-polled release does at every dispatch: query the events of blocks in flight
        for b in sorted(issue_op):
            if issue_op[b] < i and b not in seen_done and b not in pending:
                pending.append(b)
        q0 = time.perf_counter()
        for b in list(pending):
            n_query += 1
            if B.ss_batch_done(run.ctx, 0, b):
                seen_done[b] = i
                pending.remove(b)
        t_query += time.perf_counter() - q0
    t0 = time.perf_counter()
    run_iteration_dispatch(run.ctx, run.tr.n_ops, run_op, plan["points"])
    torch.cuda.synchronize()
    t_step = time.perf_counter() - t0
    ours = np.array([free_op[b] - issue_op[b] for b in sorted(issue_op)])
    stock = np.array([seen_done.get(b, run.tr.n_ops) - issue_op[b] for b in sorted(issue_op)])
    n_ops = run.tr.n_ops
    run.close()

    def dist(a):
        return {"mean": round(float(a.mean()), 1), "p50": int(np.percentile(a, 50)), "p90": int(np.percentile(a, 90)),
                "p99": int(np.percentile(a, 99)), "max": int(a.max())}
    return {"mode": "reuse-interval", "config": cfgno, "swap_out_batches": len(ours),
            "ops_per_step": n_ops, "step_ms": round(t_step * 1e3, 2),
            "device_side_release_ops": dist(ours), "host_polled_release_ops": dist(stock),
            "host_polled_event_queries_per_step": n_query,
            "host_polled_query_ms_per_step": round(t_query * 1e3, 3)}


def record_hook_overhead(B, torch, shapes=None, steps=20, warmup=5):
    """Overhead of the dispatch hook on a real PyTorch training step (the comparison of the paper's
    profiler-overhead table, Sec. 6: no profiling, Lightweight mode, Detailed mode, PyTorch's built-in
    profiler): a Llama-like decoder in plain PyTorch, bf16, AdamW; step = zero_grad, forward, loss,
    backward, optimizer step."""
    import paper_2509_11076_amd.torch_hook as H
    from workloads.torch_model import Trainer
    from torch.profiler import profile, ProfilerActivity
    shapes = shapes or {"gpu_bound": dict(layers=12, hidden=1024, heads=16, seq=1024, batch=4, vocab=32000),
                        "host_bound": dict(layers=12, hidden=256, heads=4, seq=128, batch=1, vocab=32000)}

    def timed(fn, n, w):
        for _ in range(w):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3
    out = {}
    for sname, sh in shapes.items():
        tr = Trainer(argparse.Namespace(**sh))
        rows = {}
        rows["no profiling"] = dict(ms_per_step=timed(tr.step, steps, warmup))
        cfg = B.ss_config_default()
        cfg.staging_bytes = 4096
        cfg.max_ops = 1 << 18
        cfg.max_events = 1 << 20
        ctx = B.ss_create(cfg)
        tr.hook = H
        try:
            for name, mode in (("hook, Lightweight mode", H.SS_HOOK_LIGHTWEIGHT), ("hook, Detailed mode", H.SS_HOOK_DETAILED)):
                H.ss_hook_install(ctx, mode)
                ms = timed(tr.step, steps, warmup)
                ops, ev, _ = B.ss_trace_view(ctx)
                rows[name] = dict(ms_per_step=ms, ops_per_step=len(ops), events_per_step=len(ev))
            H.ss_hook_set_mode(H.SS_HOOK_OFF)
            rows["hook installed, switched off"] = dict(ms_per_step=timed(tr.step, steps, warmup))
        finally:
            H.ss_hook_remove()
            tr.hook = None
            B.ss_destroy(ctx)
        for name, kw in (("torch.profiler, CPU activity", dict()),
                         ("torch.profiler, shapes+memory+stacks", dict(record_shapes=True, profile_memory=True, with_stack=True))):
            for _ in range(2):
                tr.step()
            torch.cuda.synchronize()
            n = max(3, steps // 4)
            with profile(activities=[ProfilerActivity.CPU], **kw):
                rows[name] = dict(ms_per_step=timed(tr.step, n, 1), steps=n)
        base = rows["no profiling"]["ms_per_step"]
        for r in rows.values():
            r["overhead_pct"] = round(100 * (r["ms_per_step"] / base - 1), 1)
            r["ms_per_step"] = round(r["ms_per_step"], 3)
        out[sname] = {"workload": "Llama-like decoder, %(layers)d layers, hidden %(hidden)d, %(heads)d heads, seq %(seq)d, "
                                  "batch %(batch)d, bf16, AdamW" % sh, "steps": steps, "warmup": warmup, "modes": rows}
        log("hook overhead, %s: %s" % (sname, {k: v["overhead_pct"] for k, v in rows.items()}))
        del tr
        torch.cuda.empty_cache()
    return {"mode": "hook-overhead", "paper_table_context": "the paper's testbed: Lightweight +0.9 %, Detailed +34.6 %, "
            "PyTorch profiler +219.7 %", "shapes": out}


def record_torch_swap(B, torch, np, shape=None, limit_frac=0.9, steps=10, warmup=3, variants=None):
    """Policies generated from the hooked trace of a real PyTorch model and executed inside that model: a Llama-like
    decoder in plain PyTorch (bf16, AdamW), one Detailed-mode iteration -> ss_generate_policy for a memory limit of
    base + limit_frac x (peak - base) -> the executor around autograd's saved-tensor hooks, tensors moved with
    ss_swap_out_from / ss_swap_in_to into blocks the caching allocator places.  variants: list of (limit_frac,
    per_phase): Eq. 1 as printed (the step time spread evenly over all operators) or applied to the forward and the
    backward pass separately (two more timestamps per iteration); the first variant
    is the record's own, the others ride along under "variants"."""
    import copy
    import paper_2509_11076_amd.torch_hook as H
    from paper_2509_11076_amd.torch_executor import TorchSwapExecutor, BlockObserver, plan_from_profile
    from workloads.torch_model import Trainer
    variants = variants or [(limit_frac, False)]
    sh = shape or dict(layers=12, hidden=1024, heads=16, seq=1024, batch=4, vocab=32000)
    # attention through plain matmul and softmax kernels: every kernel of the step is deterministic, so the loss
    # with and without swapping can be compared bit for bit (the fused attention kernels accumulate in an order
    # that changes from run to run)
    torch.backends.cuda.enable_flash_sdp(False)
    torch.backends.cuda.enable_mem_efficient_sdp(False)
    tr = Trainer(argparse.Namespace(**sh))

    def timed(n, w):
        for _ in range(w):
            tr.step()
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats()
        t0 = time.perf_counter()
        for _ in range(n):
            loss = tr.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n * 1e3, torch.cuda.max_memory_allocated(), loss.detach().clone()
    for _ in range(warmup):
        tr.step()
    snap = (copy.deepcopy(tr.model.state_dict()), copy.deepcopy(tr.opt.state_dict()))

    def restore():
        tr.model.load_state_dict(copy.deepcopy(snap[0]))
        tr.opt.load_state_dict(copy.deepcopy(snap[1]))
    ms_plain, peak_plain, loss_plain = timed(steps, 0)
    restore()
    _, _, loss_again = timed(steps, 0)           # is the step itself reproducible?  only then does bit equality mean anything
    # forward / backward / optimizer split of one step (three more events)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    tr.on_phase = lambda ph: evs[ph].record()
    evs[0].record()
    tr.step()
    tr.on_phase = None
    torch.cuda.synchronize()
    t_phase = [evs[i].elapsed_time(evs[i + 1]) * 1e-3 for i in range(3)]
    cfg = B.ss_config_default()
    cfg.staging_bytes = 0
    cfg.max_ops, cfg.max_events = 1 << 18, 1 << 20
    cfg.flags = B.SS_CFG_POLICY_POINTS
    plan_ctx = exec_ctx = None
    tr.hook = H
    link = 57e9
    results = []
    try:
        plan_ctx = B.ss_create(cfg)
        H.ss_hook_install(plan_ctx, H.SS_HOOK_DETAILED)
        restore()
        ms_detailed, _, _ = timed(max(3, steps // 2), 1)
        restore()
        tr.opt.zero_grad(set_to_none=True)
        torch.cuda.synchronize()
        base = torch.cuda.memory_stats()["requested_bytes.all.current"]
        obs = BlockObserver()
        tr.saved_hooks = lambda: torch.autograd.graph.saved_tensors_hooks(obs.pack, obs.unpack)
        tr.step()
        tr.saved_hooks = None
        torch.cuda.synchronize()
        ops, ev, _ = B.ss_trace_view(plan_ctx)
        ops, ev = ops.copy(), ev.copy()
        tab = H.ss_hook_tensor_table()
        H.ss_hook_remove()
        B.ss_destroy(plan_ctx)
        plan_ctx = None
        # Eq. 1 / Eq. 3: link bytes per operator from the step just measured
        cfg.link_bytes_per_op = max(1, int(link * ms_plain * 1e-3 / max(1, len(ops))))
        n_phase = [max(1, int(((ops["sig"] >> 16) == ph).sum())) for ph in range(3)]
        per_phase = tuple(max(1, int(link * t_phase[ph] / n_phase[ph])) for ph in range(3))
        for frac, phased in variants:
            plan_ctx = B.ss_create(cfg)
            no = B.ss_timeline_scan(plan_ctx, ev, None, len(ops), base, 1 << 62)
            limit = base + int(frac * (no["peak"] - base))
            kept, descs_out, info, ap, pol = plan_from_profile(plan_ctx, ops, tab, ev, base, limit, sh["layers"], sh["layers"],
                                                               min_bytes=1 << 20, observer=obs,
                                                               phase_bytes_per_op=per_phase if phased else None)
            B.ss_destroy(plan_ctx)
            plan_ctx = None
            r = {"limit_frac_of_activation_peak": frac, "eq1": "per phase" if phased else "as printed",
                 "memory_limit_bytes": int(limit), "generator": info, "tensors_swapped": int(len(kept)),
                 "bytes_each_way_per_step": sum(int(x) for x in kept["nbytes"]),
                 "eq1_link_bytes_per_operator": list(per_phase) if phased else int(cfg.link_bytes_per_op),
                 "median_operators_between": {"swap_out_and_release": int(np.median(kept["t_free"].astype(np.int64) - kept["t_out"])) if len(kept) else None,
                                              "swap_in_and_first_use": int(np.median(kept["t_use"].astype(np.int64) - kept["t_in"])) if len(kept) else None}}
            if len(kept):
                cfg2 = B.ss_config_default()
                cfg2.staging_bytes = max(4096, int(ap["staging_bytes"]))
                cfg2.max_ops, cfg2.max_events = cfg.max_ops, cfg.max_events
                exec_ctx = B.ss_create(cfg2)
                H.ss_hook_install(exec_ctx, H.SS_HOOK_DETAILED)
                ex = TorchSwapExecutor(torch, exec_ctx, kept, descs_out, torch.cuda.current_stream())
                tr.saved_hooks = ex.hooks
                tr.on_phase = lambda ph: ex.end_iteration() if ph == 3 else ex.poll()
                restore()
                ms_swap, peak_swap, loss_swap = timed(steps, 0)
                tr.saved_hooks = tr.on_phase = None
                H.ss_hook_remove()
                B.ss_destroy(exec_ctx)
                # where the compute stream waited: three more steps in the library's measurement mode (every
                # device-side wait charged with the time from reaching it to the end of the batch it waits for)
                cfg2.flags = B.SS_CFG_STALL_TIMING | B.SS_CFG_TIMING
                exec_ctx = B.ss_create(cfg2)
                H.ss_hook_install(exec_ctx, H.SS_HOOK_DETAILED)
                ex2 = TorchSwapExecutor(torch, exec_ctx, kept, descs_out, torch.cuda.current_stream())
                tr.saved_hooks = ex2.hooks
                tr.on_phase = lambda ph: ex2.end_iteration() if ph == 3 else ex2.poll()
                restore()
                timed(3, 0)
                tr.saved_hooks = tr.on_phase = None
                st2 = B.ss_get_stats(exec_ctx)
                nb = kept["nbytes"].astype(np.float64)
                rate = {}
                for d_, name in ((0, "d2h"), (1, "h2d")):
                    ms = B.ss_batch_ms_all(exec_ctx, d_)[:len(kept)].astype(np.float64)
                    ok = ms > 0
                    rate[name] = round(float(nb[ok].sum() / ms[ok].sum() / 1e6), 2) if ok.any() else None
                r["transfer_gbps_while_copying"] = rate
                H.ss_hook_remove()
                B.ss_destroy(exec_ctx)
                exec_ctx = None
                r["compute_stream_wait_ms_per_step"] = {"before_blocks_are_released": round(st2["stall_free_ms"] / 3, 3),
                                                        "before_first_uses": round(st2["stall_wait_in_ms"] / 3, 3)}
                r.update({"executor": dict(ex.stats), "ms_per_step_swapping": round(ms_swap, 3),
                          "overhead_vs_no_swap_pct": round(100 * (ms_swap / ms_plain - 1), 1),
                          "allocator_peak_bytes_swapping": int(peak_swap),
                          "loss_after_the_same_steps_bit_equal": bool(torch.equal(loss_plain, loss_swap)),
                          "loss_swapping": float(loss_swap)})
            results.append(r)
            log("torch model swap: limit %.2f, Eq. 1 %s: %d tensors, %.0f MB each way, %s ms/step (no swap %.1f)" % (
                frac, r["eq1"], r["tensors_swapped"], r["bytes_each_way_per_step"] / 1e6, r.get("ms_per_step_swapping"), ms_plain))
    finally:
        tr.saved_hooks = tr.on_phase = None
        H.ss_hook_remove()
        tr.hook = None
        for c in (plan_ctx, exec_ctx):
            if c is not None:
                B.ss_destroy(c)
        torch.backends.cuda.enable_flash_sdp(True)
        torch.backends.cuda.enable_mem_efficient_sdp(True)
    first = results[0]
    out = {"mode": "torch-model-swap",
           "workload": "Llama-like decoder in plain PyTorch, %(layers)d layers, hidden %(hidden)d, %(heads)d heads, seq %(seq)d, "
                       "batch %(batch)d, bf16, AdamW, attention by matmul + softmax kernels; policy generated from its own hooked "
                       "trace and executed inside it" % sh,
           "steps": steps, "ops_per_step": int(len(ops)), "allocator_events_per_step": int(len(ev)),
           "operators_per_phase": {"forward": n_phase[0], "backward": n_phase[1], "optimizer": n_phase[2]},
           "no_swap_phase_ms": {"forward": round(t_phase[0] * 1e3, 2), "backward": round(t_phase[1] * 1e3, 2),
                                "optimizer": round(t_phase[2] * 1e3, 2)},
           "ms_per_step": {"no_hook_no_swap": round(ms_plain, 3), "detailed_hook_no_swap": round(ms_detailed, 3),
                           "swapping": first.get("ms_per_step_swapping")},
           "allocator_peak_bytes": {"no_swap": int(peak_plain), "swapping": first.get("allocator_peak_bytes_swapping"),
                                    "planned_with_policy": int(first["generator"]["peak_with_policy"])},
           "loss_without_swapping_reproducible_bit_for_bit": bool(torch.equal(loss_plain, loss_again)),
           "loss": {"no_swap": float(loss_plain), "no_swap_again": float(loss_again), "swapping": first.get("loss_swapping")}}
    out.update({k: v for k, v in first.items() if k not in ("ms_per_step_swapping", "allocator_peak_bytes_swapping", "loss_swapping")})
    if len(results) > 1:
        out["variants"] = results[1:]
    return out


# ---- the fixed-sequence configurations: 1, 2, 3, 5 ----------------------------------------------------

def measure(B, torch, np, bw, o):
    """one record for configuration o.config with o.steps timed steps after o.warmup warm-up steps"""
    from workloads.harness import SwapRun
    paths = {"auto": B.SS_PATH_AUTO, "kernel": B.SS_PATH_KERNEL, "engine": B.SS_PATH_ENGINE, "staged": B.SS_PATH_STAGED}

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    cfgno = o.config
    bpo = o.bpo
    workgroups_out = o.workgroups_out
    extra = {}
    if cfgno == 3:       # 7B shape under a 48 GB budget: greedy policy, link share fixed so that it fits
        extra = dict(budget=48 * 10**9, min_bytes=1 << 20)
        if bpo <= 0:
            bpo = 256 << 20
    if o.policy_mode == "generated":
        # the paper's generator (Sec. 4) picks the swap set for a memory limit instead of the
        # configuration prescribing it; one logical layer per decoder layer and phase
        if cfgno not in (2, 3):
            sys.exit("--policy-mode generated: configurations 2 and 3 only")
        from workloads import transformer as T
        shape = T.config_shape(cfgno)
        extra = dict(min_bytes=1 << 16, generator=dict(g_fwd=shape.layers, g_bwd=shape.layers, c_num=1, c_den=1),
                     policy_points=o.timing == "policy-points")
        if cfgno == 2:
            tr_ = T.build_trace(shape)
            pcfg = B.ss_config_default()
            pcfg.staging_bytes = 4096
            sctx = B.ss_create(pcfg)
            extra["budget"] = int(o.limit_frac * B.ss_timeline_scan(sctx, tr_.events, None, tr_.n_ops, 0, 1 << 62,
                                                                    want_per_op=False)["peak"])
            B.ss_destroy(sctx)
            del tr_
        else:
            extra["budget"] = 48 * 10**9
    has_compute = cfgno != 5
    if cfgno == 5:       # small-tensor stress: no model around it
        extra = dict(compute=False)
        if bpo <= 0:
            bpo = 256 << 20
    # the same step without any swapping
    if has_compute:
        base = SwapRun(B, torch, cfgno, swap=False)
        t_noswap = timed(base.step_noswap, o.steps, o.warmup)
        base_n_ops = base.tr.n_ops
        # forward / backward split of the no-swap step (two markers): operators of the forward pass are
        # several times shorter than those of the backward pass, which Eq. 1's even spread ignores
        ph = list(base.tr.op_phase)
        first_bwd = ph.index(1) if 1 in ph else len(ph)
        ev3 = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev_op = [torch.cuda.Event(enable_timing=True) for _ in range(base.tr.n_ops)]     # one more pass, an event per operator
        ev3[0].record()
        for i in range(base.tr.n_ops):
            if i == first_bwd:
                ev3[1].record()
            base.compute.run_op(i)
            ev_op[i].record()
        if first_bwd == len(ph):
            ev3[1].record()
        ev3[2].record()
        torch.cuda.synchronize()
        t_fwd, t_bwd = ev3[0].elapsed_time(ev3[1]) * 1e-3, ev3[1].elapsed_time(ev3[2]) * 1e-3
        # no-swap time at which each operator has finished, scaled to the timed no-swap step (the events cost a little)
        t_done_noswap = np.array([ev3[0].elapsed_time(e) for e in ev_op]) * 1e-3
        t_done_noswap *= t_noswap / max(t_done_noswap[-1], 1e-9)
        del ev_op
        n_fwd, n_bwd = max(1, first_bwd), max(1, len(ph) - first_bwd)
        base.close()
        del base
        torch.cuda.empty_cache()
        log("config %d: no-swap baseline done: %.1f ms/step" % (cfgno, t_noswap * 1e3))
    else:
        t_noswap, base_n_ops = 1e-9, 1
        t_done_noswap = None
        t_fwd = t_bwd = 0.0
        n_fwd = n_bwd = 1

    # Link model.  Eq. 1 spreads the measured iteration time evenly over the operators and Eq. 3
    # turns bytes into time, so bytes-per-operator = link peak x iteration time / operators.  The
    # iteration time under swapping is not known before swapping: as in the paper's GenPolicy stage
    # (several policies are generated from successive measured iterations and the fastest is kept,
    # Sec. 6), the model is re-fitted from the measured step time a few times and the best kept.
    flags = B.SS_CFG_TIMING | (B.SS_CFG_KEEP_LATE if o.policy_mode == "execute-all" else 0)
    if getattr(o, "bare_ring", -1) == 1:
        flags |= B.SS_CFG_BARE_RING
    if getattr(o, "memory_markers", -1) == 1:
        flags |= B.SS_CFG_MEMORY_MARKERS
    link = min(bw["d2h_gbps"], bw["h2d_gbps"]) * 1e9
    calib = []
    # the swap-in queue is planned with the no-swap operator time: operators never run faster than that
    bpo_in = max(1, int(link * t_noswap / base_n_ops)) if cfgno in (1, 2) else 0
    if cfgno == 3:
        # swap-ins planned at half the swap-out share: they are issued about twice as far ahead of their use,
        # so the link starts bringing tensors back as soon as the first backward operators have freed room
        # (2.25 s -> 2.16 s per step; at 112 MiB and below the budget no longer holds them)
        bpo_in = o.bpo_in if o.bpo_in > 0 else 128 << 20
    if o.policy_mode == "generated" and o.timing == "link-model" and bpo <= 0:
        # swap-outs queue up during the forward pass, swap-ins during the backward pass: each queue gets
        # that pass's measured bytes per operator (with 10 % margin); the generator's Eq. 1 keeps the
        # whole-iteration average
        extra["generator"]["bpo"] = max(1, int(link * t_noswap / base_n_ops))
        bpo = max(1, int(0.9 * link * t_fwd / n_fwd))
        bpo_in = max(1, int(0.9 * link * t_bwd / n_bwd))
    if o.policy_mode == "generated" and o.timing == "policy-points" and o.phase_eq1 and has_compute:
        # Eq. 1 per phase: a forward operator is several times shorter than a backward one here; the
        # forward operators are cut into as many logical layers as still hold the largest candidate
        from workloads import transformer as T
        tab_ = T.build_trace(T.config_shape(cfgno)).tensors
        keep_ = (tab_["first_bwd_use"] != 0xFFFFFFFF) & (tab_["last_fwd_use"] != 0xFFFFFFFF)
        biggest = int(tab_["nbytes"][keep_].max())
        f_bpo, b_bpo = max(1, int(link * t_fwd / n_fwd)), max(1, int(link * t_bwd / n_bwd))
        extra["generator"]["phase_bytes_per_op"] = (f_bpo, b_bpo, b_bpo)
        extra["generator"]["g_fwd"] = max(1, min(extra["generator"]["g_fwd"], int(n_fwd * f_bpo // (3 * biggest // 2))))
        if bpo <= 0:
            bpo = max(1, int(link * t_noswap / base_n_ops))      # not used by the generator's own points
    path, path_in = paths[o.path], paths[o.path_in or o.path]
    window_in = o.engine_window if o.engine_window >= 0 else ((4, bw["h2d_gbps"] * 1e9, t_bwd) if has_compute else 0)

    more_cfg = {k: int(v, 0) for k, v in (kv.split("=", 1) for kv in getattr(o, "cfg", []))}

    def make(bpo_, wgo=workgroups_out, p=None, p_in=None, fl=None):
        r_ = make_(bpo_, wgo, p, p_in, fl)
        if getattr(o, "iteration_end", "drain") == "nowait":
            r_.iteration_end = B.SS_SYNC_ITERATION_END
        return r_

    def make_(bpo_, wgo, p, p_in, fl):
        return SwapRun(B, torch, cfgno, swap=True, bpo=bpo_, bpo_in=bpo_in, copy_path=path if p is None else p,
                       copy_path_in=path_in if p_in is None else p_in, copy_workgroups=o.workgroups,
                       copy_workgroups_out=wgo, flags=flags if fl is None else fl, cfg_extra=dict(copy_cus=getattr(o, "copy_cus", 0), engine_window_in=window_in, engine_window_out=o.engine_window_out, **more_cfg), **extra)

    def trial(label, **kw):
        r = make(**kw)
        t = timed(r.step, 3 if t_noswap > 0.02 else 40, 2 if t_noswap > 0.02 else 12)     # short steps: more of them
        forced, dropped = r.n_forced, r.n_dropped
        r.close()
        del r
        torch.cuda.empty_cache()
        log("config %d: %s -> %.1f ms/step" % (cfgno, label, t * 1e3))
        return t, forced, dropped
    if bpo <= 0:
        bpo = max(1, int(link * t_noswap / base_n_ops))
        for _ in range(max(1, o.calibrate)):
            t_trial, forced, dropped = trial("link-model fit, %d bytes/op" % bpo, bpo_=bpo)
            calib.append({"link_bytes_per_op": bpo, "ms_per_step": round(t_trial * 1e3, 2), "forced": forced,
                          "dropped": dropped})
            nxt = max(1, int(link * t_trial / base_n_ops))
            if any(abs(nxt - c["link_bytes_per_op"]) < 0.03 * nxt for c in calib):
                break
            bpo = nxt
        bpo = min(calib, key=lambda c: c["ms_per_step"])["link_bytes_per_op"]
    # grid of the pack launches: a grid that saturates the link delays every kernel launched beside it,
    # a small one (8 workgroups, about 3/4 of the link rate) hardly does; which wins depends on whether
    # the step is bound by the link or by the compute stream, so both are measured and the faster kept.
    # Likewise the route: directly between the blocks and the staging area (SS_PATH_AUTO), or through the
    # rings in HBM with one copy-engine transfer per ring slot (SS_PATH_STAGED).  Configuration 3's tensors
    # exceed a ring slot and all go by copy engine: nothing to choose there.
    grid_fits, path_fits, bare_fits, marker_fits = [], [], [], []
    if has_compute and cfgno != 3 and o.calibrate > 0:
        if o.path == "auto" and o.path_in is None and cfgno == 2:
            for name, p in (("auto", B.SS_PATH_AUTO), ("staged", B.SS_PATH_STAGED)):
                fl_ = flags | (B.SS_CFG_BARE_RING if p == B.SS_PATH_STAGED and getattr(o, "bare_ring", -1) != 0 else 0)
                t_trial = trial("route %s" % name, bpo_=bpo, p=p, p_in=p, fl=fl_)[0]
                path_fits.append({"route": name, "ms_per_step": round(t_trial * 1e3, 2)})
            if path_fits[1]["ms_per_step"] < 0.99 * path_fits[0]["ms_per_step"]:
                path = path_in = B.SS_PATH_STAGED
        if B.SS_PATH_STAGED in (path, path_in) and getattr(o, "bare_ring", -1) < 0:
            # the ring's copy-engine transfers with events on their stream, or bare and issued by the library's
            # own thread (SS_CFG_BARE_RING)
            for name, fl in (("with events", flags), ("bare", flags | B.SS_CFG_BARE_RING)):
                t_trial = trial("ring transfers %s" % name, bpo_=bpo, p=path, p_in=path_in, fl=fl)[0]
                bare_fits.append({"ring_transfers": name, "ms_per_step": round(t_trial * 1e3, 2)})
            if bare_fits[1]["ms_per_step"] < 0.995 * bare_fits[0]["ms_per_step"]:
                flags |= B.SS_CFG_BARE_RING
        if getattr(o, "memory_markers", -1) < 0:
            # markers of the compute stream's position: events that the swap streams wait for, or a count in device memory
            for name, fl in (("events", flags), ("device memory", flags | B.SS_CFG_MEMORY_MARKERS)):
                t_trial = trial("markers through %s" % name, bpo_=bpo, p=path, p_in=path_in, fl=fl)[0]
                marker_fits.append({"markers": name, "ms_per_step": round(t_trial * 1e3, 2)})
            if marker_fits[1]["ms_per_step"] < 0.995 * marker_fits[0]["ms_per_step"]:
                flags |= B.SS_CFG_MEMORY_MARKERS
        if workgroups_out == 0 and path != B.SS_PATH_STAGED:
            for wgo in (0, 8):
                t_trial = trial("pack grid %s" % (wgo or "default"), bpo_=bpo, wgo=wgo)[0]
                grid_fits.append({"workgroups_out": wgo or "default", "ms_per_step": round(t_trial * 1e3, 2)})
            if grid_fits[1]["ms_per_step"] < 0.98 * grid_fits[0]["ms_per_step"]:
                workgroups_out = 8
    # Bare ring transfers are timed on the host's clock, which takes a third small transfer per ring transfer and a
    # watching thread (SS_CFG_TIMING): the timed steps then run without SS_CFG_TIMING, as a user of the library would
    # run them, and the per-launch figures come from a second context with it, after the timed region.
    separate_timing = bool(flags & B.SS_CFG_BARE_RING) and B.SS_PATH_STAGED in (path, path_in)
    run = make(bpo_=bpo, wgo=workgroups_out, fl=(flags & ~B.SS_CFG_TIMING) if separate_timing else None)
    n_forced, n_dropped_setup, run_generated = run.n_forced, run.n_dropped, run.generated
    engine_window_used = run.engine_window_in
    for _ in range(o.warmup):
        run.step()
    torch.cuda.synchronize()
    st0 = B.ss_get_stats(run.ctx)
    # the timed region: nothing but the steps (per-batch events are read after it)
    t0 = time.perf_counter()
    for _ in range(o.steps):
        run.step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / o.steps
    run.iteration_end = None                # what follows reads events and the staging area: the host waits again
    st1 = B.ss_get_stats(run.ctx)
    steps_before_events = o.warmup + o.steps
    if separate_timing:
        hl_timed = run.host_ms_log[-o.steps:]
        run.close()
        del run
        torch.cuda.empty_cache()
        run = make(bpo_=bpo, wgo=workgroups_out)
        for _ in range(max(o.warmup, 10)):            # the stage machine needs nine iterations to settle
            run.step()
        torch.cuda.synchronize()
        steps_before_events = max(o.warmup, 10)
    # per-launch durations from the HIP events recorded on the swap streams: those of the last timed step,
    # and of up to three more steps run for this purpose alone
    unit_ms = {0: [], 1: [], 2: [], 3: []}
    ring_kernel_ms = {0: [], 1: []}          # gathers into / scatters out of the rings
    spans = {0: [], 1: [], 2: [], 3: []}

    def read_events():
        for d in (0, 1, 2, 3):
            ms = B.ss_batch_ms_all(run.ctx, d)
            if d < 2:            # a batch that went through a ring is timed as its gather / scatter inside HBM: not a link figure
                grp_ = B.ss_ring_view(run.ctx, d)[0]
                if len(grp_) == len(ms):
                    in_ring = ms[grp_ >= 0]
                    ring_kernel_ms[d] += in_ring[in_ring >= 0].tolist()
                    ms = ms[grp_ < 0]
            ms = ms[ms >= 0]
            if len(ms):
                unit_ms[d] += ms.tolist()
                try:
                    spans[d].append(B.ss_batch_ms(run.ctx, d)[1])
                except B.SsError:                 # first unit of the direction did not run that way
                    pass
    read_events()
    # GB/s per batch-size class (direct batches only: a batch that went through the ring is timed as its gather
    # or scatter inside HBM), from the events of the last timed step
    by_size = {}
    for d, key, st_key in ((0, "descs_out", "out_start"), (1, "descs_in", "in_start")):
        ms = B.ss_batch_ms_all(run.ctx, d)
        starts = B.ss_schedule_view(run.ctx)[d]
        csum = np.concatenate(([0], np.cumsum(run.last["applied"][key]["nbytes"].astype(np.int64))))
        nb_ = csum[starts[1:]] - csum[starts[:-1]]
        grp = B.ss_ring_view(run.ctx, d)[0]
        for b in range(len(ms)):
            if ms[b] <= 0 or (len(grp) and grp[b] >= 0) or starts[b + 1] == starts[b]:
                continue
            cls = 1 << max(0, int(nb_[b]) - 1).bit_length()           # next power of two
            e = by_size.setdefault((d, cls), [0, 0, 0.0])
            e[0] += 1; e[1] += int(nb_[b]); e[2] += float(ms[b])
    phase_ms = []                           # forward / backward pass of these steps on the compute stream (two markers)
    for _ in range(min(3, o.steps)):
        if has_compute:
            pe = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            run.before_op = lambda i, pe=pe: (pe[0].record() if i == 0 else pe[1].record() if i == first_bwd else None)
        run.step()
        if has_compute:
            pe[2].record()
        torch.cuda.synchronize()
        if has_compute and 0 < first_bwd < run.tr.n_ops:
            phase_ms.append((pe[0].elapsed_time(pe[1]), pe[1].elapsed_time(pe[2])))
        read_events()
    run.before_op = None
    event_steps = 1 + min(3, o.steps)
    st2 = B.ss_get_stats(run.ctx)
    applied, match, scan = run.last["applied"], run.last["match"], run.last["scan"]
    steps_all = steps_before_events + event_steps - 1
    lib_stats = {
        # anchors placed per matching level over all steps of this context: (token, stack, sig), (token, sig),
        # (token), sequence alignment, unmatched
        "anchors_by_match_level": dict(zip(("full_key", "token_sig", "token", "aligned", "unmatched"),
                                           [int(x) for x in st2["match_levels"]])),
        # memory-block reuse interval of the loaded schedule (Sec. 6.4): operators between issuing a tensor's
        # swap-out and the release of its block; bucket b = floor(log2(interval + 1))
        "reuse_interval_ops": {"mean": round(st2["reuse_sum"] / max(1, st2["reuse_count"]), 2),
                               "log2_histogram": [int(x) for x in st2["reuse_hist"]]},
        "free_waits_per_step": int(st2["free_waits"]) // max(1, steps_all),
        "wait_in_waits_per_step": int(st2["in_waits"]) // max(1, steps_all),
        "engine_window_waits_per_step": int(st2["engine_window_waits"]) // max(1, steps_all)}
    bytes_way = run.bytes_each_way
    assert st1["bytes_out"] - st0["bytes_out"] == o.steps * bytes_way == st1["bytes_in"] - st0["bytes_in"]
    n_ops = run.tr.n_ops
    hl = hl_timed if separate_timing else run.host_ms_log[-(o.steps + event_steps - 1):][:o.steps]
    trace_work = {k: round(sum(h[k] for h in hl) / len(hl), 3) for k in ("match", "apply", "scan")}
    n_events = len(run.tr.events)
    reused = sum(1 for h in hl if h["apply"] == 0.0)
    run.close()
    del run
    torch.cuda.empty_cache()
    # time the compute stream spends inside the device-side waits: two more steps in the library's measurement
    # mode (one more event on the compute stream before every wait; the drain joins the compute stream too)
    if has_compute and not getattr(o, "no_stall_timing", False):
        srun = SwapRun(B, torch, cfgno, swap=True, bpo=bpo, bpo_in=bpo_in, copy_path=path, copy_path_in=path_in,
                       copy_workgroups=o.workgroups, copy_workgroups_out=workgroups_out, flags=flags | B.SS_CFG_STALL_TIMING,
                       cfg_extra=dict(copy_cus=getattr(o, "copy_cus", 0), engine_window_in=window_in,
                                      engine_window_out=o.engine_window_out, **more_cfg), **extra)
        srun.step()
        torch.cuda.synchronize()
        a = B.ss_get_stats(srun.ctx)
        for _ in range(2):
            srun.step()
        torch.cuda.synchronize()
        b_ = B.ss_get_stats(srun.ctx)
        lib_stats["compute_stream_wait_ms_per_step"] = {
            "for_swap_outs_before_a_block_is_released": round((b_["stall_free_ms"] - a["stall_free_ms"]) / 2, 3),
            "for_swap_ins_before_a_first_use": round((b_["stall_wait_in_ms"] - a["stall_wait_in_ms"]) / 2, 3)}
        srun.close()
        del srun
        torch.cuda.empty_cache()

    per_step = lambda k: (st1[k] - st0[k]) // o.steps
    kernel_batches, engine_batches = per_step("kernel_batches"), per_step("engine_batches")
    engine_out = per_step("engine_batches_out")
    ring_out, ring_in = per_step("ring_batches"), per_step("ring_batches_in")
    ring_tr_out, ring_tr_in = per_step("ring_transfers"), per_step("ring_transfers_in")
    nob, nib = int(applied["n_out_batches"]), int(applied["n_in_batches"])
    engine_in = engine_batches - engine_out

    def mover(ring, engine, nb):
        if ring and ring == nb:
            return "copy kernel into the HBM ring + one copy-engine transfer per ring slot"
        if ring:
            return "mixed (ring and direct)"
        if engine == nb:
            return "copy engine"
        return "copy kernel" if engine == 0 else "mixed (copy kernel and copy engine)"
    out_by, in_by = mover(ring_out, engine_out, nob), mover(ring_in, engine_in, nib)

    value = 2 * bytes_way / t_step / 1e9
    # link-side units of a direction: the ring transfers if it went through the ring, else its batches
    # what crosses the link: the batches that move directly, and the ring transfers
    out_link_ms = unit_ms[0] + unit_ms[2]
    in_link_ms = unit_ms[1] + unit_ms[3]
    both = lambda a, b: [max(x, y) for x, y in zip(a, b)] if a and b and len(a) == len(b) else (a or b)
    out_link_span = both(spans[2], spans[0]) if ring_out else spans[0]
    in_link_span = both(spans[3], spans[1]) if ring_in else spans[1]
    gb = lambda ms_total: bytes_way * event_steps / (ms_total * 1e-3) / 1e9 if ms_total > 0 else 0.0
    d2h_busy, h2d_busy = gb(sum(out_link_ms)), gb(sum(in_link_ms))            # while a transfer / launch runs
    d2h_span = bytes_way / (np.mean(out_link_span) * 1e-3) / 1e9 if out_link_span else 0.0   # first start .. last end
    h2d_span = bytes_way / (np.mean(in_link_span) * 1e-3) / 1e9 if in_link_span else 0.0
    t_floor = max(t_noswap, bytes_way / (bw["d2h_gbps"] * 1e9), bytes_way / (bw["h2d_gbps"] * 1e9))
    # the last tensors to leave are the first needed back, so the two directions hardly overlap:
    t_floor_serial = max(t_noswap, bytes_way / (bw["d2h_gbps"] * 1e9) + bytes_way / (bw["h2d_gbps"] * 1e9))
    # ... and the schedule has two ends the link cannot help with: nothing can leave before the operator after
    # which the first swap-out is issued, and what follows the first use of the tensor that comes back last runs
    # after the last byte has arrived (both taken from the step without swapping)
    t_floor_sched = None
    if t_done_noswap is not None and len(applied["actions"]):
        a_ = applied["actions"]
        outs_, uses_ = a_["op_idx"][a_["kind"] == B.SS_ACT_OUT], a_["op_idx"][a_["kind"] == B.SS_ACT_WAIT_IN]
        if len(outs_) and len(uses_) and t_floor_serial > t_noswap:
            head = float(t_done_noswap[min(int(outs_.min()), len(t_done_noswap) - 1)])
            last_use = min(int(uses_.max()), len(t_done_noswap) - 1)
            tail = float(t_done_noswap[-1] - (t_done_noswap[last_use - 1] if last_use > 0 else 0.0))
            t_floor_sched = t_floor_serial + head + tail
    # roofline of the mover of the swap-out direction (the dominant one: it holds the forward pass back)
    if out_by == "copy kernel":
        kname, k_ms, k_peak = "ss_copy_kernel<to host>, pack launches (swap-out)", unit_ms[0], bw["d2h_gbps"]
    elif ring_out:
        kname, k_ms, k_peak = "copy-engine transfers out of the HBM ring (swap-out); gathers by ss_copy_kernel", unit_ms[2], bw["d2h_gbps"]
    else:
        kname, k_ms, k_peak = "copy engine, one hipMemcpyAsync per tensor (swap-out)", unit_ms[0], bw["d2h_gbps"]
    if k_ms:
        avg_launch_ms = sum(k_ms) / len(k_ms)
        bytes_per_launch = bytes_way * event_steps / len(k_ms)
        link_achieved = bytes_per_launch / (avg_launch_ms * 1e-3) / 1e9
    else:
        avg_launch_ms = bytes_per_launch = link_achieved = 0.0
    roof = {"bound": "host_link", "achieved": round(link_achieved, 2), "peak": round(k_peak, 2), "unit": "GB/s",
            "frac": round(link_achieved / k_peak, 4),
            "traffic": int(PACK_TRAFFIC_RATIO * 2 * bytes_per_launch) if out_by == "copy kernel" else None,
            "traffic_note": "derived, not a counter of this run: %.3f x the algorithmic bytes of a launch (HBM read + host "
                            "write = 2 x bytes_per_launch), the ratio rocprofv3 FETCH_SIZE / WRITE_SIZE gave for the pack "
                            "kernel (%s)" % (PACK_TRAFFIC_RATIO, PACK_TRAFFIC_SOURCE),
            "mover": out_by, "kernel": kname, "avg_launch_ms": round(avg_launch_ms, 4),
            "bytes_per_launch": int(bytes_per_launch), "launches_timed": len(k_ms),
            "launches_timed_note": (("HIP events of %d steps of a second context with SS_CFG_TIMING, run after the timed "
                                     "region (the timed steps run without it)" % event_steps) if separate_timing else
                                    "HIP events of the last timed step and of %d further steps" % (event_steps - 1)) + (
                "; the ring's bare copy-engine transfers carry no events and are timed on the host's clock (a copy of each "
                "transfer's sequence number arriving in pinned memory, watched by a thread that makes no HIP call)"
                if flags & B.SS_CFG_BARE_RING and B.SS_PATH_STAGED in (path, path_in) else ""),
            "hbm": {"achieved": round(link_achieved, 2), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(link_achieved / HBM_PEAK_GBPS, 5),
                    "note": "HBM side of the same bytes (one HBM access per byte moved over the link); by design far from the HBM roofline"}}
    if (ring_out and ring_kernel_ms[0]) or (ring_in and ring_kernel_ms[1]):
        g_ms = (ring_kernel_ms[0] if ring_out else []) + (ring_kernel_ms[1] if ring_in else [])
        g_bytes = bytes_way * event_steps * (int(bool(ring_out)) + int(bool(ring_in)))
        roof["ring_kernel"] = {"kernel": "ss_copy_kernel, HBM <-> HBM ring (gather / scatter)", "bound": "hbm",
                               "achieved": round(2 * g_bytes / (sum(g_ms) * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                               "unit": "GB/s", "frac": round(2 * g_bytes / (sum(g_ms) * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                               "launches_timed": len(g_ms), "avg_launch_ms": round(sum(g_ms) / len(g_ms), 4),
                               "note": "read + write bytes of the launches over their summed durations"}
    rec = {
        "metric": METRIC, "value": round(value, 3), "unit": "GB/s",
        "value_definition": "(D2H bytes + H2D bytes of a step) / step wall time; the per-direction shares of the link "
                            "peak are in pct_of_link_peak, each against that direction's own measured peak",
        "n_gpus": 1, "steps": o.steps, "warmup": o.warmup,
        "ms_per_step": round(t_step * 1e3, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": WORKLOADS[cfgno] + (" [swap set chosen by the policy generator for the memory limit instead]"
                                                   if o.policy_mode == "generated" else ""),
                   "ops_per_step": n_ops, "tensors_swapped": int(applied["n_kept"]),
                   "bytes_each_way": bytes_way, "out_batches": nob, "in_batches": nib,
                   "copy_path_out": {v: k for k, v in paths.items()}[path],
                   "copy_path_in": {v: k for k, v in paths.items()}[path_in],
                   "kernel_launches_per_step": int(kernel_batches), "engine_batches_per_step": int(engine_batches),
                   "ring_transfers_per_step": {"out": int(ring_tr_out), "in": int(ring_tr_in)},
                   "swap_out_by": out_by, "swap_in_by": in_by,
                   "link_bytes_per_op": bpo, "prefetch_bytes_per_op": bpo_in, "engine_window_in": engine_window_used,
                   "link_model_fits": calib,
                   "route_fits": path_fits, "pack_grid_fits": grid_fits, "ring_transfer_fits": bare_fits, "marker_fits": marker_fits,
                   "markers": "a count in device memory (SS_CFG_MEMORY_MARKERS)" if flags & B.SS_CFG_MEMORY_MARKERS else "events",
                   "ring_transfers": ("bare, issued by the library's own thread" if flags & B.SS_CFG_BARE_RING
                                      else "with events on their stream") if B.SS_PATH_STAGED in (path, path_in) else None,
                   "pack_workgroups": workgroups_out or o.workgroups or "default (64)", "policy_mode": o.policy_mode,
                   "timing": o.timing if o.policy_mode == "generated" else "link-model",
                   "generator_params": {k: v for k, v in extra.get("generator", {}).items()} or None,
                   "noswap_forward_ms": round(t_fwd * 1e3, 2), "noswap_backward_ms": round(t_bwd * 1e3, 2),
                   "swap_forward_ms": round(float(np.mean([p_[0] for p_ in phase_ms])), 2) if phase_ms else None,
                   "swap_backward_ms": round(float(np.mean([p_[1] for p_ in phase_ms])), 2) if phase_ms else None,
                   "memory_limit_bytes": extra.get("budget"), "generator": run_generated,
                   "memory_limit_met": (int(scan["peak"]) <= extra["budget"]) if extra.get("budget") else None,
                   "tensors_forced_late": n_forced, "tensors_dropped": n_dropped_setup, "peak_bytes_with_policy": int(scan["peak"]),
                   "stage": int(match["stage"]), "anchors_unmatched": int(match["n_unmatched"])},
        "trace_work_host_ms_per_step": dict(trace_work, steps_reusing_the_loaded_schedule=reused,
                                            note="wall time of the call incl. host<->device copies and synchronisation; "
                                                 "%d operators, %d events, %d anchors; in the Stable stage an iteration whose "
                                                 "anchors land where they did reuses the loaded schedule (apply and scan 0)"
                                                 % (n_ops, n_events, int(applied["n_kept"]) + n_dropped_setup)),
        "link_peak_measured": {k: round(v, 2) for k, v in bw.items()},
        "pct_of_link_peak": {
            "d2h_while_copying": round(100 * d2h_busy / bw["d2h_gbps"], 1),
            "h2d_while_copying": round(100 * h2d_busy / bw["h2d_gbps"], 1),
            "d2h_first_start_to_last_end": round(100 * d2h_span / bw["d2h_gbps"], 1),
            "h2d_first_start_to_last_end": round(100 * h2d_span / bw["h2d_gbps"], 1),
            "note": "each direction against its own one-direction peak; the two directions follow one another in the "
                    "step (what leaves last is needed back first), so their sum over the whole step is not comparable "
                    "with either peak"},
        "step_time": {"noswap_ms": round(t_noswap * 1e3, 3), "swap_ms": round(t_step * 1e3, 3),
                      "overhead_vs_noswap_pct": round(100 * (t_step / t_noswap - 1), 1),
                      "target_overhead_pct": 5.0,
                      "compute_stream_stall_ms": round((t_step - t_noswap) * 1e3, 3),
                      "floor_ms": round(t_floor * 1e3, 3),
                      "overhead_vs_floor_pct": round(100 * (t_step / t_floor - 1), 1),
                      "floor_out_then_in_ms": round(t_floor_serial * 1e3, 3),
                      "overhead_vs_floor_out_then_in_pct": round(100 * (t_step / t_floor_serial - 1), 1),
                      "floor_out_then_in_with_schedule_ends_ms": None if t_floor_sched is None else round(t_floor_sched * 1e3, 3),
                      "overhead_vs_floor_with_schedule_ends_pct": None if t_floor_sched is None else round(100 * (t_step / t_floor_sched - 1), 1),
                      "floor_note": "floor_out_then_in = bytes / D2H peak + bytes / H2D peak (what leaves last is needed back "
                                    "first); with_schedule_ends adds, from the step without swapping, the time before the "
                                    "operator the first swap-out follows and the time from the first use of the last "
                                    "tensor to come back to the end of the step",
                      "link_bound": bool(t_floor_serial > 1.05 * t_noswap)},
        "roofline": roof,
        "library_statistics": lib_stats,
        "gbps_by_batch_size": [{"direction": "out" if d == 0 else "in", "batch_bytes_up_to": cls, "batches": n,
                                "gbps_while_running": round(tot / (ms * 1e-3) / 1e9, 2)}
                               for (d, cls), (n, tot, ms) in sorted(by_size.items())],
    }
    if not has_compute:
        for k in ("noswap_ms", "overhead_vs_noswap_pct", "compute_stream_stall_ms", "floor_ms", "overhead_vs_floor_pct"):
            rec["step_time"][k] = None
    if not o.no_cpu_baseline and o.policy_mode != "generated":
        rec["cpu_baseline"] = cpu_baseline_safe(cfgno, bpo)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None, choices=[1, 2, 3, 4, 5],
                    help="measure this configuration alone; default: configuration 3 as the headline and the "
                         "others as sub-records")
    ap.add_argument("--no-sub-records", action="store_true", help="default mode: the headline only")
    ap.add_argument("--path", default="auto", choices=["auto", "kernel", "engine", "staged"])
    ap.add_argument("--path-in", default=None, choices=["auto", "kernel", "engine", "staged"],
                    help="copy path of the swap-in direction (default: same as --path)")
    ap.add_argument("--workgroups", type=int, default=0)
    ap.add_argument("--workgroups-out", type=int, default=0,
                    help="grid of the swap-out (pack) launches alone; 0 = same as --workgroups")
    ap.add_argument("--bpo", type=int, default=0,
                    help="link model: bytes the link moves per operator; 0 = link peak x no-swap step time / "
                         "operators per step, both measured in this run (Eq. 1 and Eq. 3 of the paper)")
    ap.add_argument("--bpo-in", type=int, default=0,
                    help="configuration 3: the same for the swap-in queue (0 = as --bpo)")
    ap.add_argument("--policy-mode", default="execute-all", choices=["execute-all", "link-aware", "generated", "staged"],
                    help="execute-all: every tensor of the prescribed set is swapped even where the link "
                         "cannot hide it; link-aware: items whose swap-out cannot finish before their "
                         "backward use are dropped; generated: the library's policy generator (Sec. 4) picks "
                         "the swap set for a memory limit (configurations 2 and 3) and its own points are kept; "
                         "staged: the loop of Algo. 1 (WarmUp without swapping, GenPolicy with a new generated "
                         "policy per iteration, Stable with the fastest of them), --steps iterations after it "
                         "settles")
    ap.add_argument("--timing", default="link-model", choices=["link-model", "policy-points"],
                    help="--policy-mode generated: release and pre-trigger points from the operator-granular link "
                         "model fed with per-phase operator times measured in this run (default), or the "
                         "generator's own logical-layer points")
    ap.add_argument("--phase-eq1", action="store_true",
                    help="--timing policy-points: Eq. 1 applied to the forward and the backward pass separately "
                         "(their measured times), with fewer forward layers; default: Eq. 1 as printed")
    ap.add_argument("--limit-frac", type=float, default=0.7,
                    help="--policy-mode generated, configuration 2: memory limit as a fraction of the no-swap peak")
    ap.add_argument("--calibrate", type=int, default=4, help="at most this many re-fits of the link model")
    ap.add_argument("--engine-window-out", type=int, default=0, help="the same for copy-engine swap-out batches")
    ap.add_argument("--memory-markers", type=int, default=-1,
                    help="1 = the compute stream's position reaches the swap streams' kernel batches through device memory "
                         "(SS_CFG_MEMORY_MARKERS), 0 = through events, -1 = both are tried and the faster kept")
    ap.add_argument("--iteration-end", default="drain", choices=["drain", "nowait"],
                    help="how a timed step ends: drain = the host waits for the swap streams (SS_SYNC_DRAIN), nowait = it "
                         "does not, the next step is ordered behind this one on the device (SS_SYNC_ITERATION_END)")
    ap.add_argument("--cfg", action="append", default=[], metavar="FIELD=VALUE",
                    help="set a further field of the library's configuration record by name (integer value), e.g. "
                         "--cfg ring_slot_bytes=134217728; may be given several times")
    ap.add_argument("--bare-ring", type=int, default=-1,
                    help="ring route: 1 = ring transfers issued bare by the library's own thread (SS_CFG_BARE_RING), "
                         "0 = with events on their stream, -1 = both are tried and the faster kept")
    ap.add_argument("--engine-window", type=int, default=-1,
                    help="copy-engine swap-in batches outstanding at most (0 = no limit): the dispatch thread waits in "
                         "ss_swap_in for the batch issued that many batches earlier; default: 4 where the swap-in bytes "
                         "need more than 1.5 x the no-swap backward pass on the link, else no limit")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-stall-timing", action="store_true",
                    help="leave out the two extra steps in the library's stall-measurement mode")
    ap.add_argument("--swap-only", action="store_true",
                    help="counter-collection mode: the same swap schedule without the compute stream's work, "
                         "no baseline, no link-model fitting (keeps a rocprofv3 --pmc run short)")
    ap.add_argument("--reuse-interval", action="store_true",
                    help="memory-block reuse interval (Sec. 6.4): operators dispatched between a tensor's swap-out "
                         "and the release of its block, with the device-side release of this library and with a "
                         "host-polled release (stock recordStream) emulated on the same run")
    ap.add_argument("--path-table", action="store_true",
                    help="GB/s of one batch of equal-size tensors at scattered arena offsets, per size class, "
                         "copy kernel against per-tensor copy-engine calls, both directions (no compute stream work)")
    ap.add_argument("--transfer-cost-table", action="store_true",
                    help="what copy-engine transfers (with and without another command on their stream) and the library's "
                         "swap-ins by engine and by kernel cost a compute stream that nothing orders against them")
    ap.add_argument("--mover-table", action="store_true",
                    help="configuration 2 with every mover per direction inside the step (copy kernel, copy engine, the "
                         "HBM rings), and what each mover costs a compute stream that does not wait for it")
    ap.add_argument("--hook-overhead", action="store_true",
                    help="overhead of the dispatch hook on a real PyTorch training step: no profiling, Lightweight, "
                         "Detailed, torch.profiler (the paper's profiler-overhead table)")
    ap.add_argument("--torch-swap", action="store_true",
                    help="a policy generated from the hooked trace of a real PyTorch model, executed inside that model "
                         "(saved-tensor hooks, blocks placed by the caching allocator); memory limit = base + --limit-frac x "
                         "(peak - base)")
    ap.add_argument("--probe-reps", type=int, default=10)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the swap executor has no inter-GPU step); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2509_11076_amd.binding as B

    torch.cuda.set_device(0)
    paths = {"auto": B.SS_PATH_AUTO, "kernel": B.SS_PATH_KERNEL, "engine": B.SS_PATH_ENGINE, "staged": B.SS_PATH_STAGED}

    def emit(line):
        print(json.dumps(line), flush=True)

    if args.hook_overhead:
        return emit(record_hook_overhead(B, torch, steps=args.steps, warmup=args.warmup))
    if args.torch_swap:
        lf = args.limit_frac if any(a.startswith("--limit-frac") for a in sys.argv) else 0.9
        return emit(record_torch_swap(B, torch, np, steps=args.steps, warmup=args.warmup,
                                      variants=[(lf, False), (lf, True), (0.95, False), (0.95, True), (0.97, True)]))

    # host-link peak, measured now (pinned hipMemcpy; 1 GiB transfers)
    pcfg = B.ss_config_default()
    pcfg.staging_bytes = 4096
    pcfg.copy_workgroups = args.workgroups
    pctx = B.ss_create(pcfg)
    bw = B.ss_bw_probe(pctx, 1 << 30, args.probe_reps)
    B.ss_destroy(pctx)
    log("link probe done: D2H %.1f GB/s, H2D %.1f GB/s" % (bw["d2h_gbps"], bw["h2d_gbps"]))

    if args.swap_only:
        return emit(run_swap_only(B, torch, args, paths[args.path], paths[args.path_in or args.path]))
    if args.path_table:
        return emit(record_path_table(B, torch, np, bw))
    if args.transfer_cost_table:
        return emit(record_transfer_cost_table(B, torch, np))
    if args.mover_table:
        return emit(record_mover_table(B, torch, np, bw, args))
    if args.reuse_interval:
        return emit(record_reuse_interval(B, torch, np, bw, args.config or 2, paths[args.path],
                                          paths[args.path_in or args.path]))
    if args.config == 4:
        return emit(record_config4(B, torch, np, cpu=not args.no_cpu_baseline))
    if args.policy_mode == "staged":
        if (args.config or 2) not in (2, 3):
            sys.exit("--policy-mode staged: configurations 2 and 3 only")
        return emit(record_staged(B, torch, bw, args.config or 2, args.limit_frac, args.steps))
    if args.config is not None:
        return emit(measure(B, torch, np, bw, args))

    # default: configuration 3 in full under the given step counts, the rest attached
    def opts(**kw):
        o = argparse.Namespace(**vars(args))
        for k, v in kw.items():
            setattr(o, k, v)
        return o
    t_all = time.perf_counter()
    try:
        head = measure(B, torch, np, bw, opts(config=3))
    except (B.SsError, RuntimeError) as e:
        # the host refuses 56.5 GB of pinned staging: the largest configuration that fits is the headline
        log("configuration 3 could not be set up (%s): configuration 2 is the headline" % e)
        torch.cuda.empty_cache()
        head = measure(B, torch, np, bw, opts(config=2))
        head["config"]["headline_note"] = "configuration 3 could not be set up on this host (%s)" % e
    if not args.no_sub_records:
        subs = {}

        def sub(name, fn):
            t0 = time.perf_counter()
            try:
                subs[name] = fn()
            except Exception as e:
                subs[name] = {"failed": "%s: %s" % (type(e).__name__, e)}
            torch.cuda.empty_cache()
            log("sub-record %s done in %.1f s" % (name, time.perf_counter() - t0))
        sub("config_1", lambda: measure(B, torch, np, bw, opts(config=1, steps=20, warmup=5)))
        if "config 3" in head["config"]["workload"]:
            # eleven warm-up steps: the stage machine of Algo. 1 needs nine iterations to reach Stable
            sub("config_2", lambda: measure(B, torch, np, bw, opts(config=2, steps=10, warmup=11)))
        sub("config_5", lambda: measure(B, torch, np, bw, opts(config=5, steps=3, warmup=1)))
        sub("config_4_planning", lambda: record_config4(B, torch, np, cpu=not args.no_cpu_baseline))
        # the generator's own release / pre-trigger points, Eq. 1 as the paper prints it
        sub("config_2_generated_policy_limit_0.97", lambda: measure(
            B, torch, np, bw, opts(config=2, steps=10, warmup=11, policy_mode="generated", limit_frac=0.97,
                                   timing="policy-points")))
        sub("config_2_generated_policy_limit_0.95", lambda: measure(
            B, torch, np, bw, opts(config=2, steps=10, warmup=11, policy_mode="generated", limit_frac=0.95,
                                   timing="policy-points")))
        sub("config_2_stage_loop_limit_0.95", lambda: record_staged(B, torch, bw, 2, 0.95, 5))
        sub("reuse_interval_config_2", lambda: record_reuse_interval(B, torch, np, bw, 2, B.SS_PATH_AUTO, B.SS_PATH_AUTO))
        sub("hook_overhead", lambda: record_hook_overhead(B, torch, steps=10, warmup=3))
        sub("torch_model_swap", lambda: record_torch_swap(B, torch, np, steps=10, warmup=3, variants=[(0.9, False), (0.95, False)]))
        def compact(r):
            """what the headline already says once (definitions, notes, the link peak) and per-iteration logs
            are left out of the sub-records; the modes run on their own (--config N, --policy-mode staged) print them"""
            if not isinstance(r, dict):
                return r
            drop = ("link_peak_measured", "value_definition", "note", "traffic_note", "launches_timed_note", "floor_note")
            out = {}
            for k, v in r.items():
                if k in drop:
                    continue
                if k == "iterations":
                    v = ([[e["stage"], round(e["ms"], 1)] for e in v] if isinstance(v, list) else
                         {m: len(rows) for m, rows in v.items()})
                    k = "iterations_stage_ms" if isinstance(v, list) else "iterations_planned"
                out[k] = compact(v)
            return out
        subs = {k: compact(v) for k, v in subs.items()}
        head["sub_records"] = subs
        head["sub_records_note"] = ("measured after the headline's timed region in the same process, each with the step "
                                    "counts its record states; whole run %.0f s" % (time.perf_counter() - t_all))
    emit(head)


if __name__ == "__main__":
    main()
