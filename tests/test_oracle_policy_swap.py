"""Pins for the oracle's link timing, policy application, greedy policy and byte round trip (CPU only)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads as W
from workloads.arena import place_tensors
from workloads.rng import SplitMix64
from test_oracle_trace_timeline import live_set_peak, tiny_trace

INSTANT = 1 << 40          # link bytes per operator so large that every transfer fits in one operator


def test_link_timing_hand_worked_case():
    # bpo = 100.  A: 250 bytes, out after op 0, used at 10.  B: 100 bytes, out after 0, used at 9.
    # C: 500 bytes, out after 2, used at 4.
    # swap-out FIFO: A occupies [100,350) -> running op 3; B [350,450) -> op 4; C [450,950) -> op 9 >= 4: invalid
    # swap-in as late as possible: A ends at 1000, starts 750 -> op 7; B must end by 750, starts 650 -> op 6
    t_free, t_in, late, valid = oracle.link_timing([0, 0, 2], [10, 9, 4], [250, 100, 500], 100)
    assert t_free == [3, 4, 9] and valid == [True, True, False]
    assert t_in[:2] == [7, 6] and late == [False, False, False]
    # D: 150 bytes out after op 0 ([100,250) -> op 2), used at 3: must start at 300 > 300-150: LATE, t_in = 3
    t_free, t_in, late, valid = oracle.link_timing([0], [3], [150], 100)
    assert (t_free, t_in, late, valid) == ([2], [3], [True], [True])


def test_link_timing_keep_late_hand_worked_case():
    # same three items as above, but C must be executed although its swap-out ends during op 9 > use at 4:
    # forced release after op 3, swap-in floor (3+1)*100 = 400 = its deadline: issued at op 4 == use, LATE
    t_free, t_in, late, valid, forced = oracle.link_timing([0, 0, 2], [10, 9, 4], [250, 100, 500], 100,
                                                           keep_late=True)
    assert t_free == [3, 4, 3] and t_in == [7, 6, 4]
    assert late == [False, False, True] and valid == [True] * 3 and forced == [False, False, True]


def test_link_timing_with_a_smaller_share_for_the_swap_in_queue():
    # out queue at 100 bytes/op as in the first case; in queue planned at 50 bytes/op:
    # A (250 B, use 10): ends 500, starts 250 -> op 5.  B (100 B, use 9): ends min(450, 250) = 250,
    # starts 150, but must not start before (t_free 4 + 1) * 50 = 250 -> LATE, op 5.
    t_free, t_in, late, valid = oracle.link_timing([0, 0], [10, 9], [250, 100], 100, bpo_in=50)
    assert t_free == [3, 4] and t_in == [5, 5] and late == [False, True] and valid == [True, True]


def test_no_swap_in_is_issued_before_the_last_swap_out():
    # X: 10 bytes, out after op 0, used at 20.  Y: 10 bytes, out after op 10 (t_free 11), used at 12.
    # The swap-in queue is planned with 1 byte per operator, so it would like to start X at op 10;
    # the last swap-out is issued after op 10, so nothing comes in before op 11: X at 11 (LATE),
    # Y cannot come in before its own release + 1 = 12 (LATE).
    t_free, t_in, late, valid = oracle.link_timing([0, 10], [20, 12], [10, 10], 100, bpo_in=1)
    assert t_free == [1, 11] and late == [True, True] and valid == [True, True]
    # ... and X, needed after Y, is not issued ahead of Y in the first-in first-out swap-in stream
    assert t_in == [12, 12]


def test_swap_in_issue_order_follows_order_of_need():
    # P: out after op 0, used at 30, 10 bytes.  Q: out after op 20 (released after 21), used at 25.
    # Planned at 1 byte/op the queue wants P at 20, then clamps both to the last swap-out (21);
    # Q cannot come before 22.  P is needed after Q, so it must not be issued before Q: 22 as well.
    t_free, t_in, late, valid = oracle.link_timing([0, 20], [30, 25], [10, 10], 100, bpo_in=1)
    assert t_free == [1, 21] and t_in == [22, 22]
    tr = W.build_trace(W.config_shape(2))
    pol = W.config_swap_set(tr, 2)
    ap = oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, 13 << 20, keep_late=True,
                             bpo_in=4 << 20)
    by_need = sorted((r[7], r[6]) for r in ap["resolved"] if not r[3] & 3)       # (t_use, t_in)
    assert all(b[1] >= a[1] for a, b in zip(by_need, by_need[1:]))
    assert oracle.schedule_check(ap, tr.tensors, tr.op_inputs, tr.op_outputs) == []


def test_keep_late_executes_the_whole_prescribed_set():
    tr = W.build_trace(W.config_shape(2))
    pol = W.config_swap_set(tr, 2)
    idx = pol["ref_op"].astype(np.int64)
    slow = 4 << 20                                  # a link that cannot keep up with every other layer
    drop = oracle.apply_policy(pol, idx, tr.tensors, slow)
    keep = oracle.apply_policy(pol, idx, tr.tensors, slow, keep_late=True)
    assert drop["n_dropped"] > 10 and keep["n_dropped"] == 0
    assert oracle.schedule_check(keep, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    forced = [r for r in keep["resolved"] if r[3] & oracle.F_FORCED]
    assert len(forced) == drop["n_dropped"]
    assert all(r[5] == r[7] - 1 and r[6] == r[7] and r[3] & oracle.F_LATE for r in forced)
    # a forced item gives no memory back: same peak as dropping it
    p_keep = oracle.timeline_scan(tr.events, keep["policy_events"], tr.n_ops, 0, 0)["peak"]
    p_drop = oracle.timeline_scan(tr.events, drop["policy_events"], tr.n_ops, 0, 0)["peak"]
    assert p_keep == p_drop


def test_link_timing_instantaneous_link():
    t_free, t_in, late, valid = oracle.link_timing([4, 4, 7], [20, 9, 9], [10**6, 10**9, 5], INSTANT)
    # the last item has no room: out after 7, released after 8, needed at 9 -> issued at 9 == use:
    # valid but late; the others move inside one operator each
    assert t_free == [5, 5, 8] and t_in == [19, 8, 9] and late == [False, False, True]
    assert valid == [True, True, True]
    t_free, t_in, late, valid = oracle.link_timing([7], [8], [5], INSTANT)
    assert valid == [False]


def instant_rule(t_out, t_use):
    """Release and pre-trigger points under a link so fast that every transfer fits inside one operator,
    written out from the rule itself (nothing here calls the oracle): a block is released after the
    operator that follows the swap-out's issue point; a swap-in is issued one operator before the use,
    but not before the last swap-out of the set has been issued, not before the item's own release, and,
    walking the items in order of need (first use, then index), never before an item needed earlier."""
    k = len(t_out)
    t_free = [t_out[i] + 1 for i in range(k)]
    after_last_out = max(t_out) + 1 if k else 0
    t_in = [max(t_use[i] - 1, after_last_out, t_free[i] + 1) for i in range(k)]
    run = 0
    for i in sorted(range(k), key=lambda i: (t_use[i], i)):
        t_in[i] = run = max(t_in[i], run)
    return t_free, t_in


@pytest.mark.parametrize("seed", range(40))
def test_link_timing_instantaneous_link_equals_the_rule(seed):
    rng = SplitMix64(seed, 41)
    k = 1 + rng.randint(9)
    t_out = [rng.randint(12) for _ in range(k)]
    # each item has room for its own round trip; uses may come before the set's last swap-out is issued
    # (then the swap-in lands after the use, which policy application later rejects) and may coincide
    t_use = [t_out[i] + 2 + rng.randint(8) for i in range(k)]
    nbytes = [1 + rng.randint(1 << 30) for _ in range(k)]
    want_free, want_in = instant_rule(t_out, t_use)
    t_free, t_in, late, valid = oracle.link_timing(t_out, t_use, nbytes, INSTANT)
    assert valid == [True] * k and t_free == want_free and t_in == want_in


def test_link_timing_instantaneous_link_rule_by_hand():
    # two items used by the same operator 12; the first leaves after operator 10 (released after 11, so not
    # back before 12), the second after operator 0 and could be back at 11 - but it is needed no earlier
    # than the first and queues behind it: 12 as well.  A third, used at 9 before the last swap-out (after
    # operator 10) has been issued, is held until 11: past its use.
    assert instant_rule([10, 0, 0], [12, 12, 9]) == ([11, 1, 1], [12, 12, 11])
    t_free, t_in, late, valid = oracle.link_timing([10, 0, 0], [12, 12, 9], [5, 5, 5], INSTANT)
    assert (t_free, t_in) == ([11, 1, 1], [12, 12, 11])
    assert late == [True, False, True]          # LATE marks the items the two floors held back, not the queueing


def applied_for(cfg, bpo, guard=0):
    tr = W.build_trace(W.config_shape(cfg))
    pol = W.config_swap_set(tr, cfg)
    place_tensors(tr.tensors, guard=guard)
    return tr, pol, oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, bpo, guard=guard)


@pytest.mark.parametrize("cfg,bpo", [(1, 64 * 1024), (1, INSTANT), (2, 8 << 20), (2, 64 << 20)])
def test_prescribed_swap_sets_give_checkable_schedules(cfg, bpo):
    tr, pol, ap = applied_for(cfg, bpo, guard=256)
    k = len(pol) - ap["n_dropped"]
    assert k > 0 and len(ap["actions"]) == 4 * k
    assert oracle.schedule_check(ap, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    # swap-out is issued at the last forward use, the wait at the first backward use (Sec. 4.3)
    tab = tr.tensors
    for (op, kind, tid, batch) in ap["actions"]:
        if kind == oracle.K_OUT:
            assert op == tab["last_fwd_use"][tid]
        if kind == oracle.K_WAIT_IN:
            assert op == tab["first_bwd_use"][tid]
    # staging: 256-aligned slots with a guard before, between and after
    offs = sorted((d[1], d[2]) for d in ap["descs_out"])
    assert offs[0][0] == 256 and all(o % 256 == 0 for o, _ in offs)
    for (o0, n0), (o1, _) in zip(offs, offs[1:]):
        assert o1 == o0 + (n0 + 255) // 256 * 256 + 256
    assert ap["staging_bytes"] == offs[-1][0] + (offs[-1][1] + 255) // 256 * 256 + 256
    # memory effect: the timeline with the emitted policy events equals the live-set definition
    away = {}
    for (op, kind, tid, batch) in ap["actions"]:
        if kind == oracle.K_FREE:
            away.setdefault(tid, [0, 0])[0] = op
        if kind == oracle.K_IN:
            away.setdefault(tid, [0, 0])[1] = op
    res = oracle.timeline_scan(tr.events, ap["policy_events"], tr.n_ops, 0, 0)
    assert np.array_equal(res["per_op"], live_set_peak(tab, away, tr.n_ops, 0))
    assert res["final"] == 0
    no = oracle.timeline_scan(tr.events, None, tr.n_ops, 0, 0)
    assert res["peak"] <= no["peak"]


@pytest.mark.parametrize("seed", range(40))
def test_random_policies_links_and_options_give_checkable_schedules(seed):
    """tiny random traces, a random subset as policy (some items unmatched, some claimed twice), a random
    link share per direction, with and without keeping late items: whatever the timing, nobody touches a
    tensor while it is away, every kept item has its four actions in causal order, staging slots are
    disjoint, and the scan with the emitted events equals the live-set definition at the emitted points"""
    rng = SplitMix64(seed, 31)
    n_ops = 14
    tab, ev = tiny_trace(seed, n_ops=n_ops, T=9)
    if seed % 2:                  # every other trace with all forward uses before all backward uses
        for i in range(len(tab)):
            tab["last_fwd_use"][i] = min(int(tab["last_fwd_use"][i]), 6)
            tab["first_bwd_use"][i] = max(int(tab["first_bwd_use"][i]), 8)
            tab["free_op"][i] = max(int(tab["free_op"][i]), int(tab["first_bwd_use"][i]))
            tab["alloc_op"][i] = tab["producer_op"][i] = min(int(tab["alloc_op"][i]), int(tab["last_fwd_use"][i]))
        ev = W.transformer.events_of(tab)
    op_in = [[] for _ in range(n_ops)]
    op_out = [[] for _ in range(n_ops)]
    for t in tab:
        tid = int(t["tensor_id"])
        op_out[int(t["producer_op"])].append(tid)
        for u in {int(t["last_fwd_use"]), int(t["first_bwd_use"]), int(t["free_op"])}:
            op_in[u].append(tid)
    rows = []
    for t in tab:
        if rng.randint(3):
            rows.append((int(t["producer_op"]), int(t["out_slot"]), int(t["tensor_id"]), 0, 0, 0, 0, 0, int(t["nbytes"])))
    if rows and rng.randint(2):
        rows.append(rows[0])                                  # the same tensor claimed twice
    pol = np.array(rows, dtype=W.POLICY_DT) if rows else np.zeros(0, dtype=W.POLICY_DT)
    idx = [r[0] if rng.randint(6) else -1 for r in rows]      # now and then an item without a match
    bpo = [64, 700, 3000, 1 << 40][rng.randint(4)]
    bpo_in = [None, 64, 900][rng.randint(3)]
    keep = bool(rng.randint(2))
    ap = oracle.apply_policy(pol, idx, tab, bpo, keep_late=keep, bpo_in=bpo_in)
    assert oracle.schedule_check(ap, tab, op_in, op_out) == []
    kept = [r for r in ap["resolved"] if not r[3] & (oracle.F_UNMATCHED | oracle.F_ORDER)]
    assert len(kept) + ap["n_dropped"] == len(rows) and len(ap["actions"]) == 4 * len(kept)
    assert len({r[2] for r in kept}) == len(kept)             # a tensor is swapped once
    phased = max(int(t["last_fwd_use"]) for t in tab) < min(int(t["first_bwd_use"]) for t in tab)
    if keep and phased:           # forward uses before backward uses: only unmatched and doubly claimed items go
        assert ap["n_dropped"] == sum(1 for i in idx if i < 0) + sum(
            1 for a, r in enumerate(rows) if idx[a] >= 0 and any(idx[b] >= 0 and rows[b][2] == r[2] for b in range(a)))
    points = {r[2]: (r[5], r[6]) for r in kept}
    res = oracle.timeline_scan(ev, ap["policy_events"], n_ops, 0, 0)
    assert np.array_equal(res["per_op"], live_set_peak(tab, points, n_ops, 0))
    assert res["final"] == 0


def test_schedule_checker_catches_planted_mistakes():
    tr, pol, ap = applied_for(1, INSTANT)
    assert oracle.schedule_check(ap, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    # a swap-in issued after its use
    bad = dict(ap)
    acts = list(ap["actions"])
    i = next(i for i, a in enumerate(acts) if a[1] == oracle.K_IN)
    acts[i] = (tr.n_ops - 1,) + acts[i][1:]
    bad["actions"] = sorted(acts, key=lambda a: (a[0], a[1]))
    assert oracle.schedule_check(bad, tr.tensors, tr.op_inputs, tr.op_outputs)
    # a block released before the tensor's last forward use
    bad = dict(ap)
    acts = list(ap["actions"])
    tid = acts[i][2]
    acts = [(0,) + a[1:] if (a[2] == tid and a[1] in (oracle.K_OUT, oracle.K_FREE)) else a for a in acts]
    bad["actions"] = sorted(acts, key=lambda a: (a[0], a[1]))
    assert oracle.schedule_check(bad, tr.tensors, tr.op_inputs, tr.op_outputs)
    # overlapping staging slots
    bad = dict(ap)
    d = list(ap["descs_out"])
    d[1] = (d[1][0], d[0][1] + 16) + d[1][2:]
    bad["descs_out"] = d
    assert oracle.schedule_check(bad, tr.tensors, tr.op_inputs, tr.op_outputs)


def test_unmatched_and_short_lived_items_are_dropped_and_counted():
    tr = W.build_trace(W.config_shape(1))
    pol = W.config_swap_set(tr, 1)
    idx = pol["ref_op"].astype(np.int64)
    idx[0] = -1                                    # matcher found no place
    idx[1] = tr.n_ops - 1                          # an operator without that output slot
    ap = oracle.apply_policy(pol, idx, tr.tensors, INSTANT)
    assert ap["n_dropped"] == 2
    assert ap["resolved"][0][3] & oracle.F_UNMATCHED and ap["resolved"][1][3] & oracle.F_UNMATCHED
    assert len(ap["actions"]) == 4 * (len(pol) - 2)
    # a link so slow that nothing leaves before it is needed again: everything dropped, nothing scheduled
    ap = oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, 16)
    assert ap["n_dropped"] == len(pol) and ap["actions"] == [] and ap["staging_bytes"] == 0
    assert all(r[3] & oracle.F_ORDER for r in ap["resolved"])


@pytest.mark.parametrize("seed", range(24))
def test_greedy_on_tiny_traces_against_brute_force(seed):
    tab, ev = tiny_trace(seed, n_ops=14, T=8)
    n_ops, base = 14, 0
    no = oracle.timeline_scan(ev, None, n_ops, base, 0)
    # reachable floor: swap everything that can be swapped
    cands = [i for i in range(len(tab)) if tab["last_fwd_use"][i] + 1 < tab["first_bwd_use"][i]]

    def peak_of(sub, t_in_at_use=False):
        # instantaneous link: released after the operator following the last forward use, back one
        # operator before the first backward use (or, at the latest, at that use itself)
        away = {i: (int(tab["last_fwd_use"][i]) + 1, int(tab["first_bwd_use"][i]) - (0 if t_in_at_use else 1)) for i in sub}
        return int(live_set_peak(tab, away, n_ops, base).max())

    subsets = [sub for r in range(len(cands) + 1) for sub in itertools.combinations(cands, r)]
    floor = min(peak_of(sub) for sub in subsets)
    budget = (floor + no["peak"]) // 2
    rows, ap = oracle.greedy_policy(tab, ev, n_ops, base, budget, INSTANT)
    chosen = [r[2] for r in rows]
    res = oracle.timeline_scan(ev, ap["policy_events"], n_ops, base, budget)
    # the points every chosen item must get under an instantaneous link, from the rule written out above
    # (not read from the oracle's output), and the oracle's points compared with them one by one
    def rule_points(ids):
        tf, ti = instant_rule([int(tab["last_fwd_use"][i]) for i in ids], [int(tab["first_bwd_use"][i]) for i in ids])
        return {i: (tf[q], ti[q]) for q, i in enumerate(ids)}
    want = rule_points(chosen)
    got = {r[2]: (r[5], r[6]) for r in ap["resolved"]}
    assert got == want and all(not r[3] & (oracle.F_UNMATCHED | oracle.F_ORDER) for r in ap["resolved"])
    # the scan's verdict on the chosen set is the brute-force (live-set) peak of that set at those points
    assert res["peak"] == int(live_set_peak(tab, want, n_ops, base).max()) <= budget
    assert all(want[i][1] <= tab["first_bwd_use"][i] for i in chosen)
    # greedy stops at the first prefix that fits: one item fewer, timed by the same rule, does not fit
    if chosen:
        assert int(live_set_peak(tab, rule_points(chosen[:-1]), n_ops, base).max()) > budget
    # with an instantaneous link the peak never rises as items are added
    peaks = [int(live_set_peak(tab, rule_points(chosen[:i]), n_ops, base).max()) for i in range(len(chosen) + 1)]
    assert peaks[0] == no["peak"] and all(b <= a for a, b in zip(peaks, peaks[1:]))
    # order: longest idle span first
    idle = [int(tab["first_bwd_use"][i]) - int(tab["last_fwd_use"][i]) for i in chosen]
    assert idle == sorted(idle, reverse=True)
    # below what any timing of any subset can reach the generator must give up (Algo. 2, error branch)
    unreachable = min(peak_of(sub, t_in_at_use=True) for sub in subsets) - 1
    with pytest.raises(oracle.Infeasible):
        oracle.greedy_policy(tab, ev, n_ops, base, unreachable, INSTANT)


def test_greedy_brings_the_7b_shape_under_its_budget():
    tr = W.build_trace(W.config_shape(3))
    budget = 48 * 10**9
    no = oracle.timeline_scan(tr.events, None, tr.n_ops, 0, budget)
    assert no["peak"] > 2 * budget * 0.95            # activations about twice the budget
    rows, ap = oracle.greedy_policy(tr.tensors, tr.events, tr.n_ops, 0, budget, 256 << 20, min_bytes=1 << 20)
    res = oracle.timeline_scan(tr.events, ap["policy_events"], tr.n_ops, 0, budget)
    assert res["peak"] <= budget and res["n_over"] == 0
    assert oracle.schedule_check(ap, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    moved = sum(d[2] for d in ap["descs_out"])
    assert moved >= no["peak"] - budget


# ------------------------------------------------------------- byte round trip
def test_round_trip_is_identity_and_touches_nothing_else():
    tr, pol, ap = applied_for(1, INSTANT, guard=256)
    arena_bytes = place_tensors(tr.tensors, guard=256)
    ap = oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, INSTANT, guard=256)
    rng = SplitMix64(1)
    arena = rng.bytes(arena_bytes)
    before = arena.copy()
    staging = np.full(ap["staging_bytes"], 0xA5, dtype=np.uint8)
    oracle.swap_out(arena, staging, ap["descs_out"])
    assert np.array_equal(arena, before)
    mask = np.ones(len(staging), bool)
    for d in ap["descs_out"]:
        assert np.array_equal(staging[d[1]:d[1] + d[2]], before[d[0]:d[0] + d[2]])
        mask[d[1]:d[1] + d[2]] = False
    assert (staging[mask] == 0xA5).all()                       # guards and padding untouched
    for d in ap["descs_out"]:                                  # blocks are released and reused
        arena[d[0]:d[0] + d[2]] = 0xEE
    oracle.swap_in(arena, staging, ap["descs_in"])
    assert np.array_equal(arena, before)


def test_round_trip_into_a_different_block_and_sparse_arena():
    descs_out = [(1000, 0, 77, 0, 0), (5000, 256, 1, 1, 0)]
    descs_in = [(9000, 0, 77, 0, 0), (200, 256, 1, 1, 0)]
    arena = SplitMix64(2).bytes(10000)
    src = arena.copy()
    staging = np.zeros(512, np.uint8)
    oracle.swap_out(arena, staging, descs_out)
    oracle.swap_in(arena, staging, descs_in)
    assert np.array_equal(arena[9000:9077], src[1000:1077]) and arena[200] == src[5000]
    keep = np.ones(10000, bool); keep[9000:9077] = False; keep[200] = False
    assert np.array_equal(arena[keep], src[keep])
    sp = oracle.SparseArena()
    sp.put(1000, src[1000:1077]); sp.put(5000, src[5000:5001])
    st2 = np.zeros(512, np.uint8)
    oracle.swap_out(sp, st2, descs_out)
    assert np.array_equal(st2, staging)
    oracle.swap_in(sp, st2, descs_in)
    assert np.array_equal(sp.read(9000, 77), src[1000:1077])
