"""GPU end-to-end: the synthetic training step with swapping on gives bit-identical compute
results to the same step with swapping off (Sec. 1: swapping costs no accuracy), with real block
reuse in a budget-sized arena and poison written over every released block."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2509_11076_amd.binding as B
    return B, torch


def run(B, torch, cfgno, swap, iters, **kw):
    from workloads.harness import SwapRun
    r = SwapRun(B, torch, cfgno, swap=swap, flags=B.SS_CFG_POISON_FREE if swap else 0, **kw)
    try:
        for _ in range(iters):
            r.step() if swap else r.step_noswap()
        chk, grad = r.compute.result()
        info = dict(arena=r.arena_bytes, bytes=r.bytes_each_way, stats=B.ss_get_stats(r.ctx),
                    plan=r.last, tr=r.tr, policy=r.policy)
        return chk, grad, info
    finally:
        r.close()


@pytest.mark.parametrize("path", [1, 2])
def test_toy_step_swap_on_equals_swap_off(env, path):
    B, torch = env
    chk0, g0, i0 = run(B, torch, 1, False, 1)
    chk1, g1, i1 = run(B, torch, 1, True, 1, bpo=64 * 1024, copy_path=path)
    assert i1["bytes"] > 1_500_000 and i1["stats"]["bytes_out"] == i1["stats"]["bytes_in"] == i1["bytes"]
    assert i1["stats"]["free_waits"] > 0 and i1["stats"]["in_waits"] > 0
    assert np.array_equal(chk0, chk1) and np.array_equal(g0, g1)
    assert i1["arena"] < i0["arena"]                     # released blocks were reused
    assert (chk0 != 0).sum() >= 20
    # the plan the library made is the oracle's
    tr, pol = i1["tr"], i1["policy"]
    ora = oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, 64 * 1024)
    from helpers import applied_as_arrays
    o = applied_as_arrays(ora)
    assert np.array_equal(i1["plan"]["applied"]["actions"].view(np.uint8), o["actions"].view(np.uint8))
    osc = oracle.timeline_scan(tr.events, ora["policy_events"], tr.n_ops, 0, 1 << 62)
    assert i1["plan"]["scan"]["peak"] == osc["peak"]


def test_toy_step_on_a_stream_of_the_callers_own(env):
    """the compute stream handed to ss_bind need not be the default one: the same step on a stream the
    caller created (default priority) gives the same results, swapping or not"""
    B, torch = env
    chk0, g0, _ = run(B, torch, 1, False, 2)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        chk1, g1, i1 = run(B, torch, 1, True, 2, bpo=64 * 1024, copy_path=1)
        side.synchronize()
    torch.cuda.current_stream().wait_stream(side)
    assert i1["stats"]["bytes_out"] == 2 * i1["bytes"] > 0 and i1["stats"]["free_waits"] > 0
    assert np.array_equal(chk0, chk1) and np.array_equal(g0, g1)


def test_1p3b_shape_three_iterations_swap_on_equals_swap_off(env):
    """configuration 2: every other layer's activations (about 3 GB) leave and return, 3 iterations"""
    B, torch = env
    chk0, g0, i0 = run(B, torch, 2, False, 3)
    chk1, g1, i1 = run(B, torch, 2, True, 3, bpo=8 << 20)
    assert 2.9e9 < i1["bytes"] < 3.3e9
    assert i1["stats"]["bytes_out"] == 3 * i1["bytes"] == i1["stats"]["bytes_in"]
    assert np.array_equal(chk0, chk1) and np.array_equal(g0, g1)
    assert i1["plan"]["match"]["similar"] and i1["plan"]["match"]["stage"] == B.SS_STAGE_GENPOLICY
    assert i1["plan"]["match"]["n_unmatched"] == 0


def test_7b_shape_small_scale_greedy_budget(env):
    """configuration 3 at reduced width (hidden 512, seq 512, 8 layers): activations about twice
    the budget, greedy policy, arena no larger than the budget allows, results unchanged"""
    B, torch = env
    from workloads.harness import SwapRun
    shape = W.ModelShape("naive", 512, 8, 8, 512, 1, 4)
    tr0 = W.build_trace(shape)
    no = oracle.timeline_scan(tr0.events, None, tr0.n_ops, 0, 0)
    budget = no["peak"] // 2
    res = []
    for swap in (False, True):
        r = SwapRun(B, torch, 3, swap=swap, trace=W.build_trace(shape), budget=budget if swap else None,
                    bpo=4 << 20, min_bytes=1 << 16, flags=B.SS_CFG_POISON_FREE if swap else 0)
        try:
            for _ in range(2):
                r.step() if swap else r.step_noswap()
            res.append((r.compute.result(), r.arena_bytes, r.last, r.policy, r.tr))
        finally:
            r.close()
    (c0, g0), a0, _, _, _ = res[0]
    (c1, g1), a1, plan, pol, tr = res[1]
    assert np.array_equal(c0, c1) and np.array_equal(g0, g1)
    assert plan["scan"]["peak"] <= budget and plan["scan"]["n_over"] == 0
    assert a1 <= budget * 1.15 and a1 < a0 * 0.65
    rows, _ = oracle.greedy_policy(tr.tensors, tr.events, tr.n_ops, 0, budget, 4 << 20, min_bytes=1 << 16)
    assert [tuple(int(x) for x in p) for p in pol.tolist()] == rows


def test_generated_policy_executes_with_unchanged_results(env):
    """Sec. 4 -> Sec. 5 on the 1.3B shape: the generator picks what to swap for a limit of 70 % of
    the no-swap peak, the executor runs that policy with its own release / pre-trigger points"""
    B, torch = env
    from workloads.harness import SwapRun
    tr0 = W.build_trace(W.config_shape(2))
    no = oracle.timeline_scan(tr0.events, None, tr0.n_ops, 0, 0)
    limit, bpo = int(no["peak"] * 0.7), 16 << 20
    gen = dict(g_fwd=24, g_bwd=24, c_num=1, c_den=1)
    chk0, g0, i0 = run(B, torch, 2, False, 2)
    r = SwapRun(B, torch, 2, swap=True, budget=limit, bpo=bpo, min_bytes=1 << 16, generator=gen,
                flags=B.SS_CFG_POISON_FREE)
    try:
        for _ in range(2):
            r.step()
        chk1, g1 = r.compute.result()
        plan, pol, arena_bytes, st = r.last, r.policy, r.arena_bytes, B.ss_get_stats(r.ctx)
        info = r.generated
    finally:
        r.close()
    assert np.array_equal(chk0, chk1) and np.array_equal(g0, g1)
    items, _ = oracle.generate_policy(tr0.tensors, no["per_op"], list(tr0.op_phase), limit, bpo, 24, 24, 1, 1, 1 << 16)
    assert [tuple(int(x) for x in p) for p in pol.tolist()] == items and len(items) > 10
    assert info["n_over_with_policy"] == 0 and plan["scan"]["peak"] == info["peak_with_policy"] <= limit
    assert plan["applied"]["n_dropped"] == 0 and arena_bytes <= limit * 1.1 < i0["arena"]
    assert st["bytes_out"] == st["bytes_in"] == 2 * sum(it[8] for it in items)


@pytest.mark.timeout(600)
def test_stage_loop_generates_selects_and_regenerates(env):
    """Algo. 1 end to end (m = 2, n = 5): three WarmUp iterations without swapping, six GenPolicy
    iterations each with a freshly generated policy, Stable with the fastest of them; a changed
    operator sequence sends the loop back to WarmUp and it settles again.  Every iteration's compute
    results equal those of the same trace without swapping."""
    B, torch = env
    from workloads.harness import StagedRun
    from workloads.compute import SyntheticCompute
    from workloads.arena import place_tensors
    shape_a = W.ModelShape("naive", 512, 8, 8, 512, 1, 4)
    shape_b = W.ModelShape("naive", 512, 8, 8, 512, 1, 4, experts0=2)      # two more operators per layer

    def trace_of(it):
        return W.build_trace(shape_a if it < 12 else shape_b)
    run = StagedRun(B, torch, trace_of, limit_frac=0.7, link_bytes_per_s=57e9, g_fwd=8, g_bwd=8, min_bytes=1 << 16,
                    flags=B.SS_CFG_POISON_FREE)
    big = torch.empty(int(place_tensors(trace_of(12).tensors) * 1.2), dtype=torch.uint8, device="cuda")
    expect = {}
    for key, it in (("a", 0), ("b", 12)):
        tr = trace_of(it)
        place_tensors(tr.tensors)
        comp = SyntheticCompute(tr, big)
        for i in range(tr.n_ops):
            comp.run_op(i)
        expect[key] = comp.result()
    try:
        log = [run.iteration(it) for it in range(23)]
    finally:
        run.close()
    W_, G, S = 0, 1, 2
    assert [e["stage"] for e in log] == [W_] * 3 + [G] * 6 + [S] * 4 + [W_] * 3 + [G] * 6 + [S]
    assert [e["similar"] for e in log] == [True] * 12 + [False] + [True] * 10
    for e in log:
        chk, grad = e["result"]
        want = expect["a" if e["it"] < 12 else "b"]
        assert np.array_equal(chk, want[0]) and np.array_equal(grad, want[1]), e["it"]
    assert all(e["bytes"] == 0 for e in log if e["stage"] == W_)
    assert all(e["bytes"] > 0 and e["unmatched"] == 0 for e in log if e["stage"] != W_ and e["it"] != 12)
    # iteration 12 ran the old policy on the new sequence: re-anchored by the aligner, still correct
    assert log[12]["bytes"] > 0
    # Stable keeps the fastest of the six candidates of its own GenPolicy stage
    for first_g, first_s in ((3, 9), (16, 22)):
        times = [log[i]["ms"] for i in range(first_g, first_g + 6)]
        assert log[first_s]["candidate"] == int(np.argmin(times))
    no_a = oracle.timeline_scan(trace_of(0).events, None, trace_of(0).n_ops, 0, 0)["peak"]
    assert all(e["peak"] <= 0.7 * no_a * 1.02 for e in log[3:12])
