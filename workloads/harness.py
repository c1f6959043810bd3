"""Benchmark / test harness: one configuration set up end to end, then stepped.

Plays the training framework around the swap executor: builds the synthetic
trace, owns the device arena (placing tensors first-fit over their residency
intervals, so released blocks are really reused), runs the synthetic compute
stream, and calls the library at the points an eager-mode dispatch loop would
(Sec. 3, Sec. 5).  It computes nothing of the method itself.
"""
import time

import numpy as np

from . import transformer as T
from .arena import place_tensors
from .layouts import ANCHOR_DT, NONE_OP
from .small_tensor import build_small_tensor_stress


class SwapRun:
    """cfgno 1..3, 5 with a fixed operator sequence (configuration 4 re-plans per iteration, see
    VaryingRun).  swap=False gives the no-swap baseline on an arena that holds everything."""

    def __init__(self, B, torch, cfgno, swap=True, bpo=64 << 20, budget=None, min_bytes=0, compute=True,
                 copy_path=0, copy_workgroups=0, flags=0, seed=2509, gemm_scale=1.0, guard=0, trace=None,
                 policy=None, engine_min_bytes=None, bpo_in=0, copy_workgroups_out=0, copy_unroll=0, copy_path_in=None, generator=None,
                 policy_points=True, reuse_delay=0, strict_limit=False, cfg_extra=None):
        from .compute import SyntheticCompute
        self.B, self.torch, self.cfgno, self.swap = B, torch, cfgno, swap
        if trace is not None:
            self.tr, pol = trace, policy
        elif cfgno == 5:
            self.tr, pol, _ = build_small_tensor_stress(seed=seed)
        else:
            self.tr = T.build_trace(T.config_shape(cfgno), seed=seed)
            pol = T.config_swap_set(self.tr, cfgno) if cfgno in (1, 2) else None
        if generator is not None:           # dict(g_fwd, g_bwd[, c_num, c_den]): the library's generator picks the set
            pol = None
            if policy_points:               # else the generator only selects; the link model times the items
                flags |= B.SS_CFG_POLICY_POINTS
        self.generated = None
        tr = self.tr
        cfg = B.ss_config_default()
        cfg.link_bytes_per_op = bpo
        cfg.prefetch_bytes_per_op = bpo_in
        cfg.copy_path = copy_path
        cfg.copy_path_in = copy_path if copy_path_in is None else copy_path_in
        cfg.copy_workgroups = copy_workgroups
        cfg.copy_workgroups_out = copy_workgroups_out
        cfg.copy_unroll = copy_unroll
        cfg.flags = flags
        cfg.guard_bytes = guard
        cfg.max_ops = max(65536, tr.n_ops)
        cfg.max_events = max(1 << 20, len(tr.events))
        if engine_min_bytes is not None:
            cfg.engine_min_bytes = engine_min_bytes
        self.engine_window_auto = None
        for k, v in (cfg_extra or {}).items():      # further fields of ss_config_t by name
            if k == "engine_window_in" and isinstance(v, tuple):
                self.engine_window_auto = v         # (window, link bytes per second, backward pass seconds): decided below
            else:
                setattr(cfg, k, v)
        self.budget = budget if budget is not None else (1 << 62)
        self.stream = torch.cuda.current_stream()

        # a probing context without staging: policy and timing do not depend on addresses
        cfg.staging_bytes = 0
        probe = B.ss_create(cfg)
        try:
            self.ops = np.stack([B.ss_intern_op(probe, tr.op_name[i], tr.op_stack[i], tr.op_dtype[i],
                                                len(tr.op_outputs[i]), tr.op_phase[i])
                                 for i in range(tr.n_ops)]) if tr.n_ops else np.zeros(0, B.OP_DT)
            if swap and pol is None and generator is not None:
                gen = dict(generator)
                gen_bpo = gen.pop("bpo", None)      # Eq. 1 of the generator may use another time per operator
                gctx = probe
                if gen_bpo:
                    cfg.link_bytes_per_op = int(gen_bpo)
                    gctx = B.ss_create(cfg)
                    cfg.link_bytes_per_op = bpo
                    for i in range(tr.n_ops):
                        B.ss_intern_op(gctx, tr.op_name[i], tr.op_stack[i], tr.op_dtype[i], len(tr.op_outputs[i]),
                                       tr.op_phase[i])
                try:
                    pol, self.generated = B.ss_generate_policy(gctx, self.ops, tr.tensors, tr.events, 0, self.budget,
                                                               min_bytes=min_bytes, **gen)
                finally:
                    if gctx is not probe:
                        B.ss_destroy(gctx)
                # the generator's simulator takes a tensor as gone right after its last forward use; the release
                # point it fixes afterwards may come later, so a finished policy can still exceed the limit at
                # some operators: the library says so in n_over_with_policy instead of failing
                if strict_limit and self.generated["n_over_with_policy"]:
                    raise RuntimeError("generated policy misses the memory limit at %d operators (peak %d > %d)"
                                       % (self.generated["n_over_with_policy"], self.generated["peak_with_policy"],
                                          self.budget))
            elif swap and pol is None:
                pol, _ = B.ss_greedy_policy(probe, tr.tensors, tr.events, tr.n_ops, 0, self.budget, min_bytes)
            if not swap:
                pol = pol[:0] if pol is not None else np.zeros(0, B.POLICY_DT)
            self.policy = pol
            self.anchors = np.zeros(len(pol), dtype=ANCHOR_DT)
            self.anchors["ref_op"] = pol["ref_op"]; self.anchors["out_slot"] = pol["out_slot"]
            ap = B.ss_apply_policy(probe, pol, pol["ref_op"].astype(np.int32), tr.tensors, allow_nomem=True)
        finally:
            B.ss_destroy(probe)
        res = ap["resolved"]
        kept = (res["flags"] & (B.SS_F_UNMATCHED | B.SS_F_ORDER)) == 0
        swapped = {int(r["tensor_id"]): (int(r["t_free"]), int(r["t_in"])) for r in res[kept]}
        if cfgno == 5 and trace is None:
            self.arena_bytes = 64 * 10**9          # placement is prescribed by the configuration
        else:
            self.arena_bytes = place_tensors(tr.tensors, swapped=swapped, guard=guard, reuse_delay=reuse_delay)
        self.n_forced = int(((res["flags"] & B.SS_F_FORCED) != 0).sum())
        self.n_dropped = int(ap["n_dropped"])
        self.staging_bytes = max(4096, int(ap["staging_bytes"]))
        cfg.staging_bytes = self.staging_bytes
        if self.engine_window_auto is not None:
            # flow control of the copy-engine swap-ins pays only where the link, not the backward pass, sets the
            # pace: there the dispatch thread may wait for transfers without starving the compute stream
            window, link_bps, t_bwd = self.engine_window_auto
            cfg.engine_window_in = window if int(ap["bytes_out"]) / link_bps > 1.5 * t_bwd else 0
        self.engine_window_in = int(cfg.engine_window_in)
        self.ctx = B.ss_create(cfg)
        # the library interns per context: same strings, same order, same integers
        for i in range(tr.n_ops):
            B.ss_intern_op(self.ctx, tr.op_name[i], tr.op_stack[i], tr.op_dtype[i], len(tr.op_outputs[i]),
                           tr.op_phase[i])
        self.arena = torch.empty(self.arena_bytes, dtype=torch.uint8, device="cuda")
        B.ss_bind(self.ctx, self.arena.data_ptr(), self.arena_bytes, self.stream.cuda_stream)
        self.compute = SyntheticCompute(tr, self.arena, seed=seed, gemm_scale=gemm_scale) if compute else None
        if self.compute is not None:
            self.compute.mark_swapped(swapped.keys())
        self.record = B.ss_trace_record_prepared(self.ctx, self.ops, tr.events)
        self.ref_ops = self.ops.copy()
        self.bytes_each_way = int(ap["bytes_out"])
        self.last = {}
        self.host_ms_log = []
        # optional callbacks of a checker: before_op(i) runs after the actions scheduled before operator i
        # and before the operator itself, after_op(i) after the operator and before the actions after it
        self.before_op = self.after_op = None
        self.reuse_stable = True
        self.iteration_end = None           # B.SS_SYNC_ITERATION_END: the host does not wait at the end of an iteration

    def close(self):
        if self.ctx is not None:
            self.B.ss_destroy(self.ctx)
            self.ctx = None
        self.arena = None
        self.compute = None

    def plan(self):
        """per-iteration trace work before the operators run: match (a3), apply (a4), scan (a2).
        In the Stable stage (Algo. 1) an iteration whose anchors land where they landed before reuses the
        schedule that is loaded (Sec. 3: Stable re-uses the existing policy): apply and scan are skipped."""
        B, tr = self.B, self.tr
        t0 = time.perf_counter()
        m = B.ss_match_sequence(self.ctx, self.ref_ops, self.ops, self.anchors, flags=B.SS_MATCH_STEP_STAGE)
        t1 = time.perf_counter()
        prev = self.last
        if (self.reuse_stable and prev and m["stage"] == B.SS_STAGE_STABLE and prev.get("tensors") is tr.tensors
                and np.array_equal(m["new_idx"], prev["match"]["new_idx"])):
            self.last = dict(prev, match=m, reused=True, host_ms=dict(match=(t1 - t0) * 1e3, apply=0.0, scan=0.0))
            self.host_ms_log.append(self.last["host_ms"])
            return self.last
        ap = B.ss_apply_policy(self.ctx, self.policy, m["new_idx"], tr.tensors)
        t2 = time.perf_counter()
        sc = B.ss_timeline_scan(self.ctx, tr.events, ap["policy_events"], tr.n_ops, 0, self.budget,
                                want_timeline=False, want_per_op=False)
        t3 = time.perf_counter()
        from paper_2509_11076_amd.executor import dispatch_points
        self.last = dict(match=m, applied=ap, scan=sc, points=dispatch_points(ap["actions"]), tensors=tr.tensors,
                         reused=False, host_ms=dict(match=(t1 - t0) * 1e3, apply=(t2 - t1) * 1e3, scan=(t3 - t2) * 1e3))
        self.host_ms_log.append(self.last["host_ms"])
        return self.last

    def step(self):
        """one training iteration: plan, then dispatch every operator with trace recording (a1) and
        the scheduled swap actions (a5-a7) around it"""
        from paper_2509_11076_amd.executor import run_iteration_dispatch
        B = self.B
        plan = self.plan()
        B.ss_trace_begin(self.ctx)
        rec, comp, pre, post = self.record, self.compute, self.before_op, self.after_op

        def run_op(i):
            rec(i)
            if pre is not None:
                pre(i)
            if comp is not None:
                comp.run_op(i)
            if post is not None:
                post(i)
        run_iteration_dispatch(self.ctx, self.tr.n_ops, run_op, plan["points"], end=self.iteration_end)

    def drain(self):
        """host waits for everything the swap streams still have (after iterations ended without waiting)"""
        self.B.ss_sync(self.ctx, self.B.SS_SYNC_DRAIN, 0)

    def step_noswap(self):
        """the same operators with no swap executor at all (baseline for the overhead figure)"""
        comp = self.compute
        for i in range(self.tr.n_ops):
            comp.run_op(i)


class VaryingRun:
    """Configuration 4: the operator sequence changes every iteration; the policy made for
    iteration 0 is re-anchored online, topped up if it no longer fits the budget, and executed.

    One planning context (no staging, never bound) holds the intern table and the stage machine;
    one executing context holds the staging area and is re-bound to the arena every iteration.
    """

    def __init__(self, B, torch, shape, budget, bpo, bpo_in=0, min_bytes=0, perturb=None, seed=2509,
                 flags=0, compute=True, gemm_scale=1.0, arena_slack=1.25, staging_slack=1.4, match_flags=0,
                 copy_path=0, copy_path_in=None, staging_bytes=None):
        self.B, self.torch, self.shape = B, torch, shape
        self.budget, self.min_bytes, self.perturb, self.seed = budget, min_bytes, perturb, seed
        self.do_compute, self.gemm_scale = compute, gemm_scale
        self.match_flags = match_flags      # e.g. SS_MATCH_ALIGN: anchors through the sequence aligner
        cfg = B.ss_config_default()
        cfg.link_bytes_per_op = bpo
        cfg.prefetch_bytes_per_op = bpo_in
        cfg.flags = flags
        cfg.copy_path = copy_path
        cfg.copy_path_in = copy_path if copy_path_in is None else copy_path_in
        cfg.staging_bytes = 0
        self.cfg = cfg
        self.plan_ctx = B.ss_create(cfg)
        tr0 = T.build_trace(shape, seed=seed, iteration=0)
        self.ref_ops = self.intern(tr0)
        pol, _ = B.ss_greedy_policy(self.plan_ctx, tr0.tensors, tr0.events, tr0.n_ops, 0, budget, min_bytes)
        self.ref_policy = pol
        self.anchors = np.zeros(len(pol), dtype=ANCHOR_DT)
        self.anchors["ref_op"] = pol["ref_op"]; self.anchors["out_slot"] = pol["out_slot"]
        ap = B.ss_apply_policy(self.plan_ctx, pol, pol["ref_op"].astype(np.int32), tr0.tensors, allow_nomem=True)
        cfg2 = B.ss_config_default()
        for f, _t in cfg._fields_:
            setattr(cfg2, f, getattr(cfg, f))
        cfg2.staging_bytes = staging_bytes or int(ap["staging_bytes"] * staging_slack) + (1 << 20)
        self.exec_ctx = B.ss_create(cfg2) if compute else None      # planning alone needs no staging
        self.staging_bytes = cfg2.staging_bytes
        self.arena = None
        self.arena_cap = int(budget * arena_slack)
        if compute:
            self.arena = torch.empty(self.arena_cap, dtype=torch.uint8, device="cuda")
        self.stream = torch.cuda.current_stream()

    def intern(self, tr):
        B = self.B
        if tr.n_ops == 0:
            return np.zeros(0, B.OP_DT)
        return np.stack([B.ss_intern_op(self.plan_ctx, tr.op_name[i], tr.op_stack[i], tr.op_dtype[i],
                                        len(tr.op_outputs[i]), tr.op_phase[i]) for i in range(tr.n_ops)])

    def close(self):
        for c in (self.plan_ctx, self.exec_ctx):
            if c is not None:
                self.B.ss_destroy(c)
        self.plan_ctx = self.exec_ctx = None
        self.arena = None

    def plan(self, it):
        """trace of iteration `it`, re-anchored policy, top-up; returns everything a checker needs"""
        B = self.B
        tr = T.build_trace(self.shape, seed=self.seed, iteration=it, perturb=self.perturb if it else None)
        ops = self.intern(tr)
        t0 = time.perf_counter()
        m = B.ss_match_sequence(self.plan_ctx, self.ref_ops, ops, self.anchors,
                                flags=B.SS_MATCH_STEP_STAGE | self.match_flags)
        t1 = time.perf_counter()
        ap = B.ss_apply_policy(self.plan_ctx, self.ref_policy, m["new_idx"], tr.tensors, allow_nomem=True)
        t2 = time.perf_counter()
        sc = B.ss_timeline_scan(self.plan_ctx, tr.events, ap["policy_events"], tr.n_ops, 0, self.budget,
                                want_per_op=False)
        t3 = time.perf_counter()
        # the kept items in this iteration's coordinates
        res = ap["resolved"]
        kept = (res["flags"] & (B.SS_F_UNMATCHED | B.SS_F_ORDER)) == 0
        cur = res[kept].copy()
        cur["ref_op"] = m["new_idx"][kept]
        cur["flags"] = 0
        cur["t_out"] = cur["t_free"] = cur["t_in"] = cur["t_use"] = 0
        topped = 0
        final = cur
        if sc["peak"] > self.budget:
            final, _ = B.ss_greedy_policy(self.plan_ctx, tr.tensors, tr.events, tr.n_ops, 0, self.budget,
                                          self.min_bytes, initial=cur)
            topped = len(final) - len(cur)
        ap2 = B.ss_apply_policy(self.plan_ctx, final, final["ref_op"].astype(np.int32), tr.tensors,
                                allow_nomem=True)
        sc2 = B.ss_timeline_scan(self.plan_ctx, tr.events, ap2["policy_events"], tr.n_ops, 0, self.budget,
                                 want_per_op=False)
        t4 = time.perf_counter()
        return dict(trace=tr, ops=ops, match=m, applied_ref=ap, scan_ref=sc, carried=cur, final=final,
                    topped=topped, applied=ap2, scan=sc2,
                    host_ms=dict(match=(t1 - t0) * 1e3, apply=(t2 - t1) * 1e3, scan=(t3 - t2) * 1e3,
                                 top_up_apply_scan=(t4 - t3) * 1e3))

    def execute(self, p, checker=None):
        """place this iteration's tensors, bind, load the schedule, run the operators with swapping.
        checker (optional): called as checker(tr, ap) once the schedule is loaded; returns (before_op,
        after_op) callbacks run around every operator on the compute stream"""
        from .compute import SyntheticCompute
        from paper_2509_11076_amd.executor import run_iteration_dispatch, dispatch_points
        B, tr = self.B, p["trace"]
        res = p["applied"]["resolved"]
        kept = (res["flags"] & (B.SS_F_UNMATCHED | B.SS_F_ORDER)) == 0
        swapped = {int(r["tensor_id"]): (int(r["t_free"]), int(r["t_in"])) for r in res[kept]}
        used = place_tensors(tr.tensors, swapped=swapped, capacity=self.arena_cap)
        B.ss_bind(self.exec_ctx, self.arena.data_ptr(), self.arena_cap, self.stream.cuda_stream)
        ap = B.ss_apply_policy(self.exec_ctx, p["final"], p["final"]["ref_op"].astype(np.int32), tr.tensors)
        comp = SyntheticCompute(tr, self.arena, seed=self.seed, gemm_scale=self.gemm_scale)
        comp.mark_swapped(swapped.keys())
        rec = B.ss_trace_record_prepared(self.exec_ctx, p["ops"], tr.events)
        B.ss_trace_begin(self.exec_ctx)
        pre, post = checker(tr, ap) if checker is not None else (None, None)

        def run_op(i):
            rec(i)
            if pre is not None:
                pre(i)
            comp.run_op(i)
            if post is not None:
                post(i)
        run_iteration_dispatch(self.exec_ctx, tr.n_ops, run_op, dispatch_points(ap["actions"]))
        return comp.result(), used, ap


class StagedRun:
    """The whole loop of Sec. 3 - Sec. 5 driven by the stage machine of Algo. 1.

    WarmUp: the iteration runs without swapping (no policy is trusted yet).  GenPolicy: every
    iteration a new policy is generated from the previous iteration's trace and its measured time
    (Eq. 1), re-anchored on the current sequence, executed and timed.  Stable: the fastest of the
    generated policies is kept (Sec. 6: with n = 5 several policies are generated and the best is
    selected) and re-anchored every iteration.  A sequence that is no longer similar sends the
    machine back to WarmUp and the candidates are dropped.

    trace_of(it) -> Trace gives iteration it's operators (what a dispatch hook would have recorded).
    """
    WARMUP, GENPOLICY, STABLE = 0, 1, 2

    def __init__(self, B, torch, trace_of, limit_frac, link_bytes_per_s, g_fwd, g_bwd, min_bytes=0, c_num=1,
                 c_den=1, seed=2509, flags=0, gemm_scale=1.0, match_flags=None, staging_bytes=None,
                 arena_bytes=None):
        self.B, self.torch, self.trace_of = B, torch, trace_of
        self.limit_frac, self.link = limit_frac, link_bytes_per_s
        self.gen = dict(g_fwd=g_fwd, g_bwd=g_bwd, c_num=c_num, c_den=c_den, min_bytes=min_bytes)
        self.seed, self.gemm_scale = seed, gemm_scale
        self.match_flags = B.SS_MATCH_ALIGN if match_flags is None else match_flags
        tr0 = trace_of(0)
        self.arena_cap = arena_bytes or int(place_tensors(tr0.tensors) * 1.3)
        self.arena = torch.empty(self.arena_cap, dtype=torch.uint8, device="cuda")
        self.cfg = B.ss_config_default()
        self.cfg.flags = flags | B.SS_CFG_POLICY_POINTS | B.SS_CFG_KEEP_LATE
        self.cfg.max_ops = max(65536, 2 * tr0.n_ops)
        self.cfg.max_events = max(1 << 20, 4 * len(tr0.events))
        self.cfg.staging_bytes = staging_bytes or int(0.6 * self.arena_cap)
        self.ctx = B.ss_create(self.cfg)
        self.stream = torch.cuda.current_stream()
        self.stage = self.WARMUP
        self.prev = None            # (trace, ops, ms, forward ms, backward ms) of the previous iteration
        self.candidates = []        # dicts(policy, ref_ops, ms, info)
        self.best = None
        self.log = []

    def close(self):
        if self.ctx is not None:
            self.B.ss_destroy(self.ctx)
            self.ctx = None
        self.arena = None

    def _intern(self, tr):
        B = self.B
        return np.stack([B.ss_intern_op(self.ctx, tr.op_name[i], tr.op_stack[i], tr.op_dtype[i],
                                        len(tr.op_outputs[i]), tr.op_phase[i]) for i in range(tr.n_ops)])

    def _generate(self):
        """a policy from the previous iteration's trace, Eq. 1 fed with its measured time"""
        B = self.B
        tr, ops, ms, ms_fwd, ms_bwd = self.prev
        no = B.ss_timeline_scan(self.ctx, tr.events, None, tr.n_ops, 0, 1 << 62, want_per_op=False)
        limit = int(self.limit_frac * no["peak"])
        self.cfg.link_bytes_per_op = max(1, int(self.link * ms * 1e-3 / max(1, tr.n_ops)))
        # the generator reads the link share from the context: a short-lived one with this iteration's value
        cfg = B.ss_config_default()
        cfg.staging_bytes = 0
        cfg.link_bytes_per_op = self.cfg.link_bytes_per_op
        cfg.max_ops, cfg.max_events = self.cfg.max_ops, self.cfg.max_events
        g = B.ss_create(cfg)
        # the generator's open constants (layer counts, C of Eq. 2) are varied around the given ones; all
        # candidates are checked against the limit in one batched scan and the best one is run
        sets = []
        for div in (1, 2, 4):
            for c_mul in (1, 4):
                d = dict(self.gen)
                d["g_fwd"] = max(1, d["g_fwd"] // div)
                d["g_bwd"] = max(1, d["g_bwd"] // div)
                d["c_num"] = d["c_num"] * c_mul
                sets.append(d)
        # Every other candidate applies Eq. 1 to the forward and the backward pass separately (their
        # measured times): the operators of the two passes differ several times in length, which the
        # even spread over the whole iteration ignores.  Which kind wins is decided by the measured
        # step time in the Stable stage.
        per_phase = len(self.candidates) % 2 == 1 and ms_fwd > 0 and ms_bwd > 0
        if per_phase:
            ph = np.asarray(tr.op_phase)
            n_fwd, n_bwd = max(1, int((ph == 0).sum())), max(1, int((ph != 0).sum()))
            f_bpo = max(1, int(self.link * ms_fwd * 1e-3 / n_fwd))
            b_bpo = max(1, int(self.link * ms_bwd * 1e-3 / n_bwd))
            tab = tr.tensors
            both = (tab["first_bwd_use"] != NONE_OP) & (tab["last_fwd_use"] != NONE_OP)
            biggest = int(tab["nbytes"][both].max()) if both.any() else 1
            for d in sets:
                d["phase_bytes_per_op"] = (f_bpo, b_bpo, b_bpo)
                # a forward layer must still hold the largest candidate's transfer
                d["g_fwd"] = max(1, min(d["g_fwd"], int(n_fwd * f_bpo // (3 * biggest // 2))))
        try:
            pol, info, chosen = B.ss_generate_policy_best(g, ops, tr.tensors, tr.events, 0, limit, sets)
        finally:
            B.ss_destroy(g)
        return dict(policy=pol, ref_ops=ops, ms=None, info=info, limit=limit, params=sets[chosen],
                    link_bytes_per_op=cfg.link_bytes_per_op, per_phase=per_phase)

    def iteration(self, it):
        from .compute import SyntheticCompute
        from paper_2509_11076_amd.executor import run_iteration_dispatch, dispatch_points
        B, torch = self.B, self.torch
        tr = self.trace_of(it)
        ops = self._intern(tr)
        stage = self.stage
        cand = None
        if stage == self.GENPOLICY and self.prev is not None:
            cand = self._generate()
            self.candidates.append(cand)
        elif stage == self.STABLE:
            if self.best is None:
                self.best = min(self.candidates, key=lambda c: c["ms"])
            cand = self.best
        unmatched = 0
        if cand is not None and len(cand["policy"]):
            pol = cand["policy"]
            anchors = np.zeros(len(pol), dtype=ANCHOR_DT)
            anchors["ref_op"] = pol["ref_op"]; anchors["out_slot"] = pol["out_slot"]
            m = B.ss_match_sequence(self.ctx, cand["ref_ops"], ops, anchors, flags=self.match_flags)
            new_idx, unmatched = m["new_idx"], int(m["n_unmatched"])
        else:
            pol, new_idx = np.zeros(0, B.POLICY_DT), np.zeros(0, np.int32)
        # placement needs the release / pre-trigger points: a dry application first
        place_tensors(tr.tensors)
        dry = B.ss_apply_policy(self.ctx, pol, new_idx, tr.tensors, allow_nomem=True)
        res = dry["resolved"]
        kept = (res["flags"] & (B.SS_F_UNMATCHED | B.SS_F_ORDER)) == 0
        swapped = {int(r["tensor_id"]): (int(r["t_free"]), int(r["t_in"])) for r in res[kept]}
        used = place_tensors(tr.tensors, swapped=swapped, capacity=self.arena_cap)
        B.ss_bind(self.ctx, self.arena.data_ptr(), self.arena_cap, self.stream.cuda_stream)
        ap = B.ss_apply_policy(self.ctx, pol, new_idx, tr.tensors)
        sc = B.ss_timeline_scan(self.ctx, tr.events, ap["policy_events"], tr.n_ops, 0, 1 << 62, want_per_op=False)
        comp = SyntheticCompute(tr, self.arena, seed=self.seed, gemm_scale=self.gemm_scale)
        comp.mark_swapped(swapped.keys())
        rec = B.ss_trace_record_prepared(self.ctx, ops, tr.events)
        points = dispatch_points(ap["actions"])
        phases = list(tr.op_phase)
        first_bwd = phases.index(1) if 1 in phases else -1
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(3)]    # start, first backward operator, end
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        B.ss_trace_begin(self.ctx)
        marks[0].record()

        def run_op(i):
            if i == first_bwd:
                marks[1].record()
            rec(i)
            comp.run_op(i)
        run_iteration_dispatch(self.ctx, tr.n_ops, run_op, points)
        marks[2].record()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
        ms_fwd = marks[0].elapsed_time(marks[1]) if first_bwd >= 0 else 0.0
        ms_bwd = marks[1].elapsed_time(marks[2]) if first_bwd >= 0 else 0.0
        if stage == self.GENPOLICY and cand is not None:
            cand["ms"] = ms
        cand_no = None if cand is None else [i for i, c in enumerate(self.candidates) if c is cand][0]
        # Algo. 1: the finished iteration's sequence against the previous one decides the next stage
        prev_ops = self.prev[1] if self.prev is not None else ops
        v = B.ss_match_sequence(self.ctx, prev_ops, ops, None, flags=B.SS_MATCH_STEP_STAGE)
        if not v["similar"]:
            self.candidates, self.best = [], None
        self.stage = int(v["stage"])
        self.prev = (tr, ops, ms, ms_fwd, ms_bwd)
        entry = dict(it=it, stage=stage, next_stage=self.stage, similar=bool(v["similar"]), ms=ms,
                     n_items=int(ap["n_kept"]), bytes=int(ap["bytes_out"]), unmatched=unmatched, peak=int(sc["peak"]),
                     arena_used=int(used),
                     candidate=cand_no, per_phase=None if cand is None else bool(cand.get("per_phase")),
                     result=comp.result())
        self.log.append(entry)
        return entry
