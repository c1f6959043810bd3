"""Boundary pins of the oracle: hand-worked cases placed exactly where an off-by-one, a strict
comparison turned non-strict, a swapped minimum / maximum or a wrong batch index would show.  Found
by planting such mistakes in oracle/ one at a time and looking for those no test noticed.  CPU only."""
import numpy as np
import pytest

import oracle
from oracle.generator import Infeasible, F_LATE
import workloads as W
from test_oracle_trace_timeline import live_set_peak
from test_oracle_generator import table

BIG = 1 << 40


# ------------------------------------------------------------------ timeline
def test_canonical_order_inside_one_operator():
    """policy allocation, trace allocations, trace frees, policy free - whatever the order of the lists"""
    ev = [(0, 1, 100), (1, 2, -20), (1, 3, 30), (2, 1, -80)]       # the release listed before the allocation
    pe = [(1, 9, -10), (1, 8, 50)]
    res = oracle.timeline_scan(ev, pe, 3, 7, 156)
    # operator 0: 107; operator 1: +50 (policy), +30 (trace), -20 (trace), -10 (policy); operator 2: -80
    assert res["timeline"].tolist() == [107, 157, 187, 167, 157, 77]
    assert res["per_op"].tolist() == [107, 187, 157] and res["final"] == 77 and res["argpeak_op"] == 1
    assert res["mre"].tolist() == [0, 31, 1] and res["n_over"] == 2          # an excess of one byte counts


def test_flag_and_stage_values_are_the_interface_ones():
    assert (oracle.F_UNMATCHED, oracle.F_ORDER, oracle.F_LATE, oracle.F_RESIZED, oracle.F_FORCED) == (1, 2, 4, 8, 16)
    assert (oracle.K_IN, oracle.K_WAIT_IN, oracle.K_OUT, oracle.K_FREE) == (0, 1, 2, 3)
    assert (oracle.WARMUP, oracle.GENPOLICY, oracle.STABLE) == (0, 1, 2)


# ------------------------------------------------------------------ link timing
def test_release_point_when_the_last_byte_lands_exactly_at_an_operator_boundary():
    # 100 link bytes per operator; the transfer starts when operator 1 starts and is 100 bytes long:
    # it fills operator 1 exactly, so the block is released after operator 1, not 2
    t_free, t_in, late, valid = oracle.link_timing([0], [5], [100], 100)
    assert (t_free, t_in, late, valid) == ([1], [4], [False], [True])
    t_free, _, _, _ = oracle.link_timing([0], [5], [101], 100)          # one byte more spills into operator 2
    assert t_free == [2]
    # the swap-in may start at the very first link byte after the release point without being late
    t_free, t_in, late, valid = oracle.link_timing([0], [3], [100], 100)
    assert (t_free, t_in, late) == ([1], [2], [False])
    t_free, t_in, late, valid = oracle.link_timing([0], [3], [101], 100)
    assert (t_free, valid) == ([2], [False]) or (t_free, t_in, late) == ([2], [3], [True])


# ------------------------------------------------------------------ policy application
def rows_for(tab):
    return np.array([(int(t["producer_op"]), int(t["out_slot"]), int(t["tensor_id"]), 0, 0, 0, 0, 0, int(t["nbytes"]))
                     for t in tab], dtype=W.POLICY_DT)


def abc():
    """A: last forward use 2, first backward use 10; B: 2 .. 9; C: 3 .. 9 (producers 0, 1, 2)"""
    tab = table([(0, 2, 10, 11, 1000), (1, 2, 9, 11, 2000), (2, 3, 9, 11, 3000)])
    tab["dev_off"] = [0, 4096, 8192]
    tab["dev_off_in"] = tab["dev_off"]
    return tab


def test_batches_batch_fields_and_swap_in_dependencies_by_hand():
    tab = abc()
    pol = rows_for(tab)
    ap = oracle.apply_policy(pol, [0, 1, 2], tab, BIG)
    # instantaneous link: released one operator after the last forward use; no swap-in before the last
    # swap-out is issued (operator 4 on); as late as possible: A before 9, then C and B before 8
    assert [r[4:8] for r in ap["resolved"]] == [(2, 3, 9, 10), (2, 3, 8, 9), (3, 4, 8, 9)]
    # swap-out batches: A and B leave after operator 2 together, C after operator 3
    assert ap["out_batch_start"] == [0, 2, 3] and [d[3] for d in ap["descs_out"]] == [0, 1, 2]
    # swap-in batches: B and C (issued before 8, used by 9), then A; the first needs both swap-out batches
    assert ap["in_batch_start"] == [0, 2, 3] and [d[3] for d in ap["descs_in"]] == [1, 2, 0]
    assert ap["in_dep"] == [1, 0]
    batch_of = {(a[1], a[2]): a[3] for a in ap["actions"]}
    assert [batch_of[(oracle.K_OUT, t)] for t in (0, 1, 2)] == [0, 0, 1]
    assert [batch_of[(oracle.K_FREE, t)] for t in (0, 1, 2)] == [0, 0, 1]
    assert [batch_of[(oracle.K_IN, t)] for t in (0, 1, 2)] == [1, 0, 0]
    assert [batch_of[(oracle.K_WAIT_IN, t)] for t in (0, 1, 2)] == [1, 0, 0]
    # staging slots in swap-out order, 256-aligned
    assert [d[1] for d in ap["descs_out"]] == [0, 1024, 3072] and ap["staging_bytes"] == 6144
    assert oracle.schedule_check(ap, tab, [[]] * 12, [[]] * 12) == []


def test_swap_in_floor_is_the_operator_after_the_last_swap_out_and_slots_round_up():
    # X: last forward use 1, first backward use 7; Y: 5 .. 9.  The last swap-out is issued after operator 5,
    # so swap-ins start at operator 6 at the earliest: X's as-late-as-possible point is exactly 6, not late
    tab = table([(0, 1, 7, 8, 257), (1, 5, 9, 10, 1)])
    ap = oracle.apply_policy(rows_for(tab), [0, 1], tab, BIG)
    assert [r[3:8] for r in ap["resolved"]] == [(0, 1, 2, 6, 7), (0, 5, 6, 8, 9)]
    # 257 bytes take two 256-byte units of staging, 1 byte one
    assert [d[1] for d in ap["descs_out"]] == [0, 512] and ap["staging_bytes"] == 768


def test_policy_events_put_an_allocation_before_a_release_of_the_same_operator():
    tab = table([(0, 2, 8, 9, 100), (1, 6, 10, 11, 200)])
    pts = rows_for(tab)
    pts[0] = (0, 0, 0, 0, 2, 5, 7, 8, 100)
    pts[1] = (1, 0, 1, 0, 6, 7, 9, 10, 200)
    ap = oracle.apply_policy(pts, [0, 1], tab, BIG, policy_points=True)
    assert ap["policy_events"] == [(5, 0, -100), (7, 0, 100), (7, 1, -200), (9, 1, 200)]


def test_resized_flag_and_point_boundaries():
    tab = abc()
    pol = rows_for(tab)
    pol["nbytes"][1] = 1999                                    # the tensor grew since the policy was made
    ap = oracle.apply_policy(pol, [0, 1, 2], tab, BIG)
    assert [r[3] & oracle.F_RESIZED for r in ap["resolved"]] == [0, oracle.F_RESIZED, 0]
    assert ap["resolved"][1][8] == 2000                        # the current size is what moves
    # the policy's own points: release at the last forward use itself and swap-in at the use are allowed,
    # release point == swap-in point is not
    pts = rows_for(tab)
    for a, (tf, ti) in enumerate([(2, 10), (5, 5), (3, 9)]):
        t = tab[a]
        pts[a] = (int(t["producer_op"]), 0, a, 0, int(t["last_fwd_use"]), tf, ti, int(t["first_bwd_use"]), int(t["nbytes"]))
    ap = oracle.apply_policy(pts, [0, 1, 2], tab, BIG, policy_points=True)
    assert [bool(r[3] & oracle.F_ORDER) for r in ap["resolved"]] == [False, True, False]
    assert ap["resolved"][0][4:8] == (2, 2, 10, 10) and ap["resolved"][2][4:8] == (3, 3, 9, 9) and ap["n_dropped"] == 1


def test_schedule_checker_names_each_planted_mistake():
    tab = abc()
    ap = oracle.apply_policy(rows_for(tab), [0, 1, 2], tab, BIG)
    reads = [[] for _ in range(12)]
    none = [[] for _ in range(12)]

    def problems(**change):
        bad = dict(ap)
        bad.update(change)
        return oracle.schedule_check(bad, tab, change.pop("reads", reads) if "reads" in change else reads, none)

    assert problems() == []
    # touching a tensor at its release operator or at its swap-in operator is fine, one operator inside is not
    for op, ok in ((3, True), (9, True), (4, False), (8, False)):
        r = [[] for _ in range(12)]
        r[op] = [0]                                            # tensor A is away strictly between 3 and 9
        got = oracle.schedule_check(ap, tab, r, none)
        assert (got == []) == ok and (ok or "while it is swapped out" in got[0])
    # staging slots that share one byte
    d = list(ap["descs_out"])
    d[1] = (d[1][0], d[0][1] + d[0][2] - 1) + d[1][2:]
    din = [x if x[3] != d[1][3] else (x[0], d[1][1]) + x[2:] for x in ap["descs_in"]]
    got = problems(descs_out=d, descs_in=din)
    assert len(got) == 1 and "overlap" in got[0]
    d[1] = (d[1][0], d[0][1] + d[0][2]) + d[1][2:]             # touching, not overlapping (then C's slot moves too)
    d[2] = (d[2][0], d[1][1] + d[1][2]) + d[2][2:]
    din = [(x[0], {y[3]: y[1] for y in d}[x[3]]) + x[2:] for x in ap["descs_in"]]
    assert problems(descs_out=d, descs_in=din) == []
    # release point == swap-in point
    acts = [(3,) + a[1:] if (a[1] == oracle.K_IN and a[2] == 1) else a for a in ap["actions"]]
    got = problems(actions=sorted(acts, key=lambda a: (a[0], a[1])))
    assert any("order violated" in g for g in got)
    # batch boundaries that do not partition the descriptors
    for starts in ([1, 2, 3], [0, 2, 2, 3], [0, 2], [0, 3, 2, 3]):
        got = problems(out_batch_start=starts)
        assert any("out batches" in g for g in got), starts
    # an action that names another batch than the one holding its descriptor; a dependency that is too early
    acts = [a[:3] + (1,) if (a[1] == oracle.K_OUT and a[2] == 0) else a for a in ap["actions"]]
    assert any("batch" in g for g in problems(actions=acts))
    assert any("depend" in g for g in problems(in_dep=[0, 0]))
    # a swap-out batch mixing two issue points
    assert any("batch" in g for g in problems(out_batch_start=[0, 3]))


# ------------------------------------------------------------------ swap
def test_sparse_arena_round_trip_from_slots_that_do_not_start_at_zero():
    sp = oracle.SparseArena()
    a, b = np.arange(77, dtype=np.uint8), np.array([200, 201, 202], dtype=np.uint8)
    sp.put(1000, a); sp.put(5000, b)
    staging = np.zeros(1024, np.uint8)
    oracle.swap_out(sp, staging, [(1000, 256, 77, 0, 0), (5000, 512, 3, 1, 0)])
    assert np.array_equal(staging[256:333], a) and np.array_equal(staging[512:515], b) and staging.sum() == a.sum() + b.sum()
    oracle.swap_in(sp, staging, [(9000, 256, 77, 0, 0), (64, 512, 3, 1, 0)])
    assert np.array_equal(sp.read(9000, 77), a) and len(sp.blocks[9000]) == 77
    assert np.array_equal(sp.read(64, 3), b) and len(sp.blocks[64]) == 3


# ------------------------------------------------------------------ matcher and aligner
def test_landings_on_operator_zero_and_anchor_beyond_the_reference():
    ops = [(1, 7, 0x101, 1), (2, 7, 0x101, 1), (3, 7, 0x101, 2)]
    idx, lvl = oracle.match_anchors(ops, ops, [(0, 0), (2, 1), (3, 0), (2, 2)])     # output 2 of a 2-output operator: none
    assert idx.tolist() == [0, 2, -1, -1] and lvl.tolist() == [0, 0, 255, 255]
    m = oracle.match_sequence(ops, ops, [(0, 0), (2, 1), (3, 0)])
    assert m["n_unmatched"] == 1 and m["new_idx"].tolist() == [0, 2, -1]
    al = oracle.align_anchors(ops, ops, [(0, 0), (2, 1), (3, 0), (2, 2)])
    assert al["new_idx"].tolist() == [0, 2, -1, -1] and al["lcs"] == 3


# ------------------------------------------------------------------ generator
def spike_case(p, size=300, lf=2, fb=12, spike=200):
    """8 forward + 8 backward operators; X (size bytes) used last forward at lf, first backward at fb,
    alive 0..13; a temporary of `spike` bytes alive during operator p only; limit = size + spike - 100"""
    tab = table([(0, lf, fb, 13, size), (p, p, W.NONE_OP, p, spike)])
    mem = live_set_peak(tab, {}, 16, 0)
    return tab, mem, [0] * 8 + [1] * 8, size + spike - 100


def test_a_tensor_relieves_operators_strictly_after_the_one_following_its_last_forward_use():
    # last forward use 2: the swap-out is issued after operator 2 and the block released after operator 3
    # at the earliest, so an excess at operator 3 is out of reach, one at operator 4 is not
    tab, mem, phases, limit = spike_case(3)
    with pytest.raises(Infeasible):
        oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64)
    tab, mem, phases, limit = spike_case(4)
    items, info = oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64)
    # one operator per layer: use in layer 12, the excess in layer 4: layers 11 .. 5 are searched downwards
    assert items == [(0, 0, 0, 0, 2, 3, 11, 12, 300)] and info["residual"] == {}
    # an excess at the first backward use itself is out of reach too; the last operator that can be
    # relieved is the one before the swap-in layer
    for p in (12, 11):
        tab, mem, phases, limit = spike_case(p)
        with pytest.raises(Infeasible):
            oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64)
    tab, mem, phases, limit = spike_case(10)
    items, _ = oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64)
    assert items == [(0, 0, 0, 0, 2, 3, 11, 12, 300)]


def test_a_layer_takes_a_transfer_only_if_strictly_more_time_remains():
    tab, mem, phases, limit = spike_case(6)
    # every layer (one operator) owns exactly the transfer's 300 link bytes: no room anywhere, both
    # directions fall back and the item is LATE
    items, _ = oracle.generate_policy(tab, mem, phases, limit, 300, 64, 64)
    assert items == [(0, 0, 0, F_LATE, 2, 10, 11, 12, 300)]
    # one link byte more per operator: swap-in in layer 11, swap-out in the last forward use's own layer
    # (released after the operator following the last forward use)
    items, _ = oracle.generate_policy(tab, mem, phases, limit, 301, 64, 64)
    assert items == [(0, 0, 0, 0, 2, 3, 11, 12, 300)]
    # forward layers with exactly 300, backward layers with 301: the swap-out has to wait for the
    # first backward layer (operator 8)
    items, _ = oracle.generate_policy(tab, mem, phases, limit, (300, 301, 301), 64, 64)
    assert items == [(0, 0, 0, 0, 2, 8, 11, 12, 300)]
    # the other way round: no backward layer (11 .. 8) takes the swap-in, the search goes on down to the
    # layer after the excess and finds the forward layer 7; the swap-out fits the last forward use's layer
    items, _ = oracle.generate_policy(tab, mem, phases, limit, (301, 300, 300), 64, 64)
    assert items == [(0, 0, 0, 0, 2, 3, 7, 12, 300)]


def test_swap_in_search_visits_every_layer_on_its_way_down():
    # two tensors of 300 bytes, both needed; 301 link bytes per one-operator layer.  The first takes the
    # layer before the use (11) and leaves 1 byte there; the second finds the next layer down (10).
    # Swap-outs likewise: the layer of the last forward use (2) has no operator after that use, so layer 3
    # takes the first (released after operator 3) and layer 4 the second (released after operator 4)
    tab = table([(0, 2, 12, 13, 300), (1, 2, 12, 13, 300), (6, 6, W.NONE_OP, 6, 500)])
    mem = live_set_peak(tab, {}, 16, 0)
    items, info = oracle.generate_policy(tab, mem, [0] * 8 + [1] * 8, 650, 301, 64, 64)
    assert items == [(0, 0, 0, 0, 2, 3, 11, 12, 300), (1, 0, 1, 0, 2, 4, 10, 12, 300)]
    assert [L[3] for L in info["layers"]][2:5] == [301, 1, 1] and [L[3] for L in info["layers"]][10:12] == [1, 1]


def test_fallback_layer_when_use_and_last_forward_use_sit_in_neighbouring_layers():
    # layers of 4 operators; X: last forward use 1 (layer 0), first backward use 6 (layer 1); excess at
    # operator 3 only; a link of 10 bytes per operator has room nowhere.  Fallback: the layer before the
    # use is layer 0, but not before the layer after the last forward use: layer 1, swap-in before
    # operator 4; release after the last operator of layer 0
    tab = table([(0, 1, 6, 7, 300), (3, 3, W.NONE_OP, 3, 200)])
    mem = live_set_peak(tab, {}, 8, 0)
    items, info = oracle.generate_policy(tab, mem, [0] * 4 + [1] * 4, 400, 10, 1, 1)
    assert items == [(0, 0, 0, F_LATE, 1, 3, 4, 6, 300)] and info["residual"] == {}


def test_minimum_size_is_inclusive_and_tensors_spanning_no_excess_are_no_candidates():
    tab, mem, phases, limit = spike_case(6)
    items, _ = oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64, min_bytes=300)
    assert len(items) == 1
    with pytest.raises(Infeasible):
        oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64, min_bytes=301)
    # Y is kept from forward to backward but idles over no excess operator: not in the candidate list
    tab = table([(0, 2, 12, 13, 300), (6, 6, W.NONE_OP, 6, 200), (7, 7, 9, 10, 50)])
    mem = live_set_peak(tab, {}, 16, 0)
    _, info = oracle.generate_policy(tab, mem, phases, int(mem.max()) - 100, BIG, 64, 64)
    assert info["rounds"] == [[0]]


def test_eq2_normalises_size_by_the_largest_candidate():
    """P: 100 bytes, spans ten excess operators; Q: 300 bytes, spans one.  Eq. 2 with C = 1:
    P 10/10 + 100/300, Q 1/10 + 300/300: P first.  (Normalised by the smallest size it would be Q.)"""
    phases = [0] * 12 + [1] * 12
    tab = table([(0, 0, 23, 23, 100), (0, 12, 15, 16, 300), (5, 5, W.NONE_OP, 14, 500)])
    mem = live_set_peak(tab, {}, 24, 0)
    limit = 850                                                # 900 over operators 5 .. 14
    assert [t for t in range(24) if mem[t] > limit] == list(range(5, 15))
    _, info = oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64)
    assert info["rounds"][0] == [0, 1]
    _, info = oracle.generate_policy(tab, mem, phases, limit, BIG, 64, 64, c_num=20, c_den=1)
    assert info["rounds"][0] == [1, 0]                         # a large C lets size win


def test_n_mre_counts_excess_operators_strictly_inside_the_idle_span():
    """excess at operators 5 .. 14.  With C = 0 only the count decides, ties go to the larger tensor.
    V idles over 6 .. 14 (last forward use 4: operator 5 is out of reach), U over 5 .. 13 (first
    backward use 14): nine each, so the larger of the two comes first, whichever it is."""
    phases = [0] * 12 + [1] * 12
    for size_u, size_v, first in ((100, 200, 2), (200, 100, 1)):
        tab = table([(0, 0, 23, 23, 50), (0, 0, 14, 15, size_u), (0, 4, 23, 23, size_v), (5, 5, W.NONE_OP, 14, 500)])
        mem = live_set_peak(tab, {}, 24, 0)
        _, info = oracle.generate_policy(tab, mem, phases, int(mem.max()) - 40, BIG, 64, 64, c_num=0, c_den=1)
        assert info["rounds"][0][0] == 0 and info["rounds"][0][1] == first     # tensor 0 spans all ten


def test_greedy_candidates_idle_over_an_over_budget_operator_and_minimum_size_is_inclusive():
    # X idles longest but only over operators within the budget; Y idles over the over-budget operator 10
    tab = table([(0, 0, 6, 7, 100), (7, 8, 12, 13, 100), (10, 10, W.NONE_OP, 10, 500)])
    ev = W.transformer.events_of(tab)
    mem = live_set_peak(tab, {}, 14, 0)
    assert [t for t in range(14) if mem[t] > 550] == [10]
    rows, ap = oracle.greedy_policy(tab, ev, 14, 0, 550, BIG)
    assert [r[2] for r in rows] == [1] and ap["resolved"][0][4:8] == (8, 9, 11, 12)
    # the minimum size is inclusive
    rows, _ = oracle.greedy_policy(tab, ev, 14, 0, 550, BIG, min_bytes=100)
    assert len(rows) == 1
    with pytest.raises(oracle.Infeasible):
        oracle.greedy_policy(tab, ev, 14, 0, 550, BIG, min_bytes=101)


def test_items_without_room_between_their_uses_and_empty_schedules():
    tab = table([(0, 3, 3, 5, 100), (1, 3, 4, 5, 100)])         # used forward and backward by the same operator; by neighbours
    ap = oracle.apply_policy(rows_for(tab), [0, 1], tab, BIG)
    assert [bool(r[3] & oracle.F_ORDER) for r in ap["resolved"]] == [True, True] and ap["n_dropped"] == 2
    assert ap["actions"] == [] and ap["out_batch_start"] == [0] and ap["in_batch_start"] == [0]
    assert oracle.schedule_check(ap, tab, [[]] * 6, [[]] * 6) == []
    # a tensor that is never used again after the forward pass, one never used in it: nothing to swap for
    tab = table([(0, 2, W.NONE_OP, 5, 100), (1, W.NONE_OP, 4, 5, 100), (2, 2, 5, 5, 100)])
    ap = oracle.apply_policy(rows_for(tab), [0, 1, 2], tab, BIG)
    assert [bool(r[3] & oracle.F_ORDER) for r in ap["resolved"]] == [True, True, False] and ap["n_dropped"] == 2
    tab = abc()                                                 # points on the uses themselves pass the checker
    pts = rows_for(tab)
    for a in range(3):
        t = tab[a]
        pts[a] = (int(t["producer_op"]), 0, a, 0, 0, int(t["last_fwd_use"]), int(t["first_bwd_use"]), 0, int(t["nbytes"]))
        pts[a]["t_out"], pts[a]["t_use"] = int(t["last_fwd_use"]), int(t["first_bwd_use"])
    ap = oracle.apply_policy(pts, [0, 1, 2], tab, BIG, policy_points=True)
    assert ap["n_dropped"] == 0 and oracle.schedule_check(ap, tab, [[]] * 12, [[]] * 12) == []


def test_equal_parameter_sets_keep_the_lower_index():
    tab, mem, phases, limit = spike_case(6)
    ev = W.transformer.events_of(tab)
    sets = [dict(g_fwd=64, g_bwd=64), dict(g_fwd=64, g_bwd=64)]
    items, chosen, _ = oracle.generate_policy_best(tab, ev, 16, 0, phases, limit, BIG, sets)
    assert chosen == 0 and len(items) == 1
