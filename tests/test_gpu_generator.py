"""GPU parity of the policy generator (Sec. 4: Eq. 1-3, Algo. 2) and of applying a generated
policy with its own release / pre-trigger points, against the oracle: exact equality."""
import numpy as np
import pytest

import oracle
import workloads as W
from workloads.arena import place_tensors
from helpers import record_lib, assert_applied_equal
from test_oracle_trace_timeline import tiny_trace, live_set_peak
from test_oracle_generator import table

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2509_11076_amd.binding as B
    return B


def make_ctx(P, **kw):
    cfg = P.ss_config_default()
    cfg.max_ops = 1 << 16
    cfg.max_events = 1 << 20
    for k, v in kw.items():
        setattr(cfg, k, v)
    return P.ss_create(cfg)


def ops_with_phases(phases):
    ops = np.zeros(len(phases), dtype=W.OP_DT)
    ops["op_token"] = 1
    ops["sig"] = [oracle.make_sig(1, 1, p) for p in phases]
    ops["n_out"] = 1
    return ops


def rows_of(pol):
    return [tuple(int(x) for x in r) for r in pol.tolist()]


def policy_events_of(items):
    pe = []
    for it in items:
        pe += [(it[5], it[2], -it[8]), (it[6], it[2], it[8])]
    return sorted(pe, key=lambda e: e[0])


def check_against_oracle(P, c, ops, phases, tab, ev, n_ops, limit, bpo, g_fwd, g_bwd, c_num=1, c_den=1, min_bytes=0,
                         per_phase=None):
    """runs both; returns the oracle's items, or None when both report infeasibility.
    per_phase: link bytes per forward / backward / optimizer operator (0 = bpo)"""
    mem = oracle.timeline_scan(ev, None, n_ops, 0, limit)["per_op"]
    obpo = bpo if per_phase is None else tuple(b or bpo for b in per_phase)
    try:
        items, info = oracle.generate_policy(tab, mem, phases, limit, obpo, g_fwd, g_bwd, c_num, c_den, min_bytes)
    except oracle.generator.Infeasible:
        with pytest.raises(P.SsError) as e:
            P.ss_generate_policy(c, ops, tab, ev, 0, limit, g_fwd, g_bwd, c_num, c_den, min_bytes, per_phase)
        assert e.value.code == P.SS_E_INFEASIBLE
        return None
    pol, res = P.ss_generate_policy(c, ops, tab, ev, 0, limit, g_fwd, g_bwd, c_num, c_den, min_bytes, per_phase)
    assert rows_of(pol) == items
    assert res["n_items"] == len(items) and res["n_rounds"] == len(info["rounds"])
    assert res["n_late"] == sum(1 for it in items if it[3] & oracle.F_LATE)
    assert res["bytes"] == sum(it[8] for it in items)
    assert res["peak_no_swap"] == max(0, int(mem.max())) if n_ops else True
    after = oracle.timeline_scan(ev, policy_events_of(items), n_ops, 0, limit)
    assert res["peak_with_policy"] == after["peak"] and res["n_over_with_policy"] == after["n_over"]
    return items


def test_hand_worked_case(P):
    """the case worked by hand in the oracle's pins: items and their four points"""
    phases = [0] * 12 + [1] * 12
    tab = table([(0, 1, 22, 23, 250), (1, 2, 20, 21, 100), (9, 10, 13, 14, 40), (8, 8, W.NONE_OP, 15, 300)])
    ev = W.transformer.events_of(tab)
    c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=100)
    try:
        pol, res = P.ss_generate_policy(c, ops_with_phases(phases), tab, ev, 0, 400, 4, 4)
        assert rows_of(pol) == [(0, 0, 0, 0, 1, 5, 18, 22, 250), (1, 0, 1, 0, 2, 8, 15, 20, 100)]
        assert res["peak_no_swap"] == 690 and res["n_rounds"] == 1 and res["bytes"] == 350
        # A is gone from operator 6 on, B from operator 9 on (operator 8 holds 650 - 250 = 400, not over the
        # limit), pre-triggers 15 and 18 after operator 14
        assert res["peak_with_policy"] <= 400 and res["n_over_with_policy"] == 0
        check_against_oracle(P, c, ops_with_phases(phases), phases, tab, ev, 24, 400, 100, 4, 4)
        # forward operators three times shorter than the average: A is released inside the peak
        slow_fwd = check_against_oracle(P, c, ops_with_phases(phases), phases, tab, ev, 24, 400, 100, 4, 4,
                                        per_phase=(34, 166, 100))
        assert {it[2]: (it[5], it[6]) for it in slow_fwd} == {0: (14, 18), 1: (5, 15)}
    finally:
        P.ss_destroy(c)


@pytest.mark.parametrize("seed", range(6))
def test_tiny_traces_limits_links_and_layer_counts(P, seed):
    n_ops = 16
    tab, _ = tiny_trace(seed, n_ops=n_ops, T=9)
    phases = [0] * 8 + [1] * 7 + [2]
    for i in range(len(tab)):
        tab["last_fwd_use"][i] = min(int(tab["last_fwd_use"][i]), 5)
        tab["first_bwd_use"][i] = min(max(int(tab["first_bwd_use"][i]), 10), 14)
        tab["free_op"][i] = max(int(tab["free_op"][i]), int(tab["first_bwd_use"][i]))
    ev = W.transformer.events_of(tab)
    ops = ops_with_phases(phases)
    peak = int(live_set_peak(tab, {}, n_ops, 0).max())
    seen = set()
    for bpo in (1 << 40, 4096, 700):
        c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo)
        try:
            for frac in (1.0, 0.95, 0.9, 0.8, 0.7, 0.5):
                for g in ((8, 7), (3, 2), (1, 1)):
                    for cnum, cden in ((1, 1), (0, 1), (7, 2)):
                        items = check_against_oracle(P, c, ops, phases, tab, ev, n_ops, int(peak * frac), bpo,
                                                     g[0], g[1], cnum, cden)
                        seen.add(None if items is None else len(items))
                    # Eq. 1 per phase: forward operators a third, backward ones twice the link share
                    check_against_oracle(P, c, ops, phases, tab, ev, n_ops, int(peak * frac), bpo, g[0], g[1],
                                         per_phase=(max(1, bpo // 3), 2 * bpo, 0))
        finally:
            P.ss_destroy(c)
    assert None in seen and 0 in seen and len(seen) >= 4   # infeasible, nothing to do, real policies


def test_edge_cases(P):
    c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=1000)
    try:
        tab = table([(0, 1, 6, 7, 500), (1, 2, 5, 6, 500)])
        ev = W.transformer.events_of(tab)
        ops = ops_with_phases([0] * 4 + [1] * 4)
        # nothing over the limit: empty policy
        pol, res = P.ss_generate_policy(c, ops, tab, ev, 0, 5000, 2, 2)
        assert len(pol) == 0 and res["n_rounds"] == 0 and res["peak_with_policy"] == res["peak_no_swap"] == 1000
        # min_bytes removes every candidate
        with pytest.raises(P.SsError) as e:
            P.ss_generate_policy(c, ops, tab, ev, 0, 600, 2, 2, min_bytes=501)
        assert e.value.code == P.SS_E_INFEASIBLE
        # zero layer counts and a zero denominator are argument errors
        for kw in (dict(g_fwd=0, g_bwd=1), dict(g_fwd=1, g_bwd=0), dict(g_fwd=1, g_bwd=1, c_den=0)):
            with pytest.raises(P.SsError) as e:
                P.ss_generate_policy(c, ops, tab, ev, 0, 600, **kw)
            assert e.value.code == P.SS_E_INVAL
        # no operators at all
        pol, res = P.ss_generate_policy(c, ops[:0], tab[:0], ev[:0], 0, 0, 1, 1)
        assert len(pol) == 0 and res["n_items"] == 0
    finally:
        P.ss_destroy(c)


@pytest.mark.parametrize("cfgno,frac,bpo,g", [(1, 0.8, 64 * 1024, 4), (2, 0.75, 16 << 20, 24), (2, 0.6, 64 << 20, 48),
                                              (3, 0.7, 256 << 20, 32)])
def test_transformer_shapes_generate_apply_and_scan(P, cfgno, frac, bpo, g):
    """Sec. 4 end to end on the transformer traces: record -> generate -> apply (policy's own points)
    on the next, perturbed iteration -> scan; every stage equal to the oracle's"""
    shape = W.config_shape(cfgno)
    tr = W.build_trace(shape)
    no = oracle.timeline_scan(tr.events, None, tr.n_ops, 0, 0)
    limit = int(no["peak"] * frac)
    c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo, flags=P.SS_CFG_POLICY_POINTS)
    try:
        ops, ev, _ = record_lib(P, c, tr)
        phases = [int(s) >> 16 for s in ops["sig"]]
        assert phases == list(tr.op_phase)
        items = check_against_oracle(P, c, ops, phases, tr.tensors, ev, tr.n_ops, limit, bpo, g, g, 1, 1, 1 << 16)
        assert items, "limit below the peak must need a policy"
        pol, res = P.ss_generate_policy(c, ops, tr.tensors, ev, 0, limit, g, g, 1, 1, 1 << 16)
        assert res["n_over_with_policy"] == 0 and res["peak_with_policy"] <= limit
        # the forward pass five times faster than the backward pass, fewer forward layers
        check_against_oracle(P, c, ops, phases, tr.tensors, ev, tr.n_ops, limit, bpo, max(1, g // 4), g, 1, 1, 1 << 16,
                             per_phase=(bpo // 3, bpo * 5 // 3, bpo))

        # same sequence: identity mapping; points kept exactly
        idx = pol["ref_op"].astype(np.int64)
        place_tensors(tr.tensors)
        ora = oracle.apply_policy(pol, idx, tr.tensors, bpo, policy_points=True)
        lib = P.ss_apply_policy(c, pol, idx, tr.tensors, allow_nomem=True)
        cmp_applied(lib, ora)
        kept = {r[2]: r for r in ora["resolved"] if not r[3] & (oracle.F_UNMATCHED | oracle.F_ORDER)}
        for it in items:
            r = kept[it[2]]
            assert (r[4], r[5], r[7]) == (it[4], it[5], it[7]) and r[6] >= it[6]
        assert oracle.schedule_check(ora, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    finally:
        P.ss_destroy(c)


def cmp_applied(lib, ora):
    from helpers import applied_as_arrays
    o = applied_as_arrays(ora)
    for key in ("resolved", "actions", "descs_out", "descs_in", "policy_events"):
        assert np.array_equal(lib[key].view(np.uint8), o[key].view(np.uint8)), key
    assert lib["staging_bytes"] == ora["staging_bytes"] and lib["n_dropped"] == ora["n_dropped"]


@pytest.mark.parametrize("keep", [False, True])
def test_generated_policy_on_varying_sequence(P, keep):
    """configuration 4's kind of change (operators dropped / inserted, lengths jittered): the policy
    generated on one iteration is re-anchored on the next and applied with its own points shifted"""
    shape = W.config_shape(2)
    tr0 = W.build_trace(shape, seed=3, iteration=0, perturb=dict(p_drop=0.05, p_insert=0.05, moe_max=8, seq_jitter=0.1))
    tr1 = W.build_trace(shape, seed=3, iteration=1, perturb=dict(p_drop=0.05, p_insert=0.05, moe_max=8, seq_jitter=0.1))
    bpo = 32 << 20
    no = oracle.timeline_scan(tr0.events, None, tr0.n_ops, 0, 0)
    flags = P.SS_CFG_POLICY_POINTS | (P.SS_CFG_KEEP_LATE if keep else 0)
    c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo, flags=flags)
    try:
        ops0, ev0, _ = record_lib(P, c, tr0)
        pol, _ = P.ss_generate_policy(c, ops0, tr0.tensors, ev0, 0, int(no["peak"] * 0.7), 24, 24, 1, 1, 1 << 16)
        assert len(pol) > 8
        ops1, _, _ = record_lib(P, c, tr1)
        anchors = np.zeros(len(pol), dtype=W.ANCHOR_DT)
        anchors["ref_op"] = pol["ref_op"]; anchors["out_slot"] = pol["out_slot"]
        m = P.ss_match_sequence(c, ops0, ops1, anchors)
        assert m["similar"] and 0 < m["n_unmatched"] < len(pol) or m["n_unmatched"] == 0
        place_tensors(tr1.tensors)
        ora = oracle.apply_policy(pol, m["new_idx"], tr1.tensors, bpo, keep_late=keep, policy_points=True)
        lib = P.ss_apply_policy(c, pol, m["new_idx"], tr1.tensors, allow_nomem=True)
        cmp_applied(lib, ora)
        assert oracle.schedule_check(ora, tr1.tensors, tr1.op_inputs, tr1.op_outputs) == []
        if keep:
            assert ora["n_dropped"] == sum(1 for r in ora["resolved"] if r[3] & (oracle.F_UNMATCHED | oracle.F_ORDER))
    finally:
        P.ss_destroy(c)


def test_best_of_several_parameter_sets_with_one_batched_scan(P):
    """ss_generate_policy_best against the oracle's selection: the hand-worked trace at three link
    speeds, and the 1.3B shape over a grid of layer counts and values of C"""
    phases = [0] * 12 + [1] * 12
    tab = table([(0, 1, 22, 23, 250), (1, 2, 20, 21, 100), (9, 10, 13, 14, 40), (8, 8, W.NONE_OP, 15, 300)])
    ev = W.transformer.events_of(tab)
    ops = ops_with_phases(phases)
    cases = [(100, [dict(g_fwd=4, g_bwd=4, min_bytes=1000), dict(g_fwd=1, g_bwd=1), dict(g_fwd=4, g_bwd=4),
                    dict(g_fwd=4, g_bwd=4, c_num=0)], 2),
             (80, [dict(g_fwd=4, g_bwd=4), dict(g_fwd=3, g_bwd=3), dict(g_fwd=3, g_bwd=4)], 1),
             (90, [dict(g_fwd=4, g_bwd=6), dict(g_fwd=4, g_bwd=4)], 1)]
    for bpo, sets, want in cases:
        c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo)
        try:
            items, chosen, info = oracle.generate_policy_best(tab, ev, 24, 0, phases, 400, bpo, sets)
            pol, res, got = P.ss_generate_policy_best(c, ops, tab, ev, 0, 400, sets)
            assert got == chosen == want and rows_of(pol) == items
            assert (res["peak_with_policy"], res["n_over_with_policy"], res["n_late"], res["bytes"]) == \
                (info["peak"], info["n_over"], info["n_late"], info["bytes"])
            with pytest.raises(P.SsError) as e:
                P.ss_generate_policy_best(c, ops, tab, ev, 0, 400, [dict(g_fwd=4, g_bwd=4, min_bytes=1000)])
            assert e.value.code == P.SS_E_INFEASIBLE
        finally:
            P.ss_destroy(c)
    tr = W.build_trace(W.config_shape(2))
    no = oracle.timeline_scan(tr.events, None, tr.n_ops, 0, 0)
    sets = [dict(g_fwd=g, g_bwd=g2, c_num=cn, c_den=2, min_bytes=1 << 16)
            for g in (6, 12, 24, 48) for g2 in (12, 24) for cn in (0, 2, 8)]
    for frac, bpo in ((0.8, 8 << 20), (0.6, 32 << 20)):
        limit = int(no["peak"] * frac)
        c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo)
        try:
            ops, ev, _ = record_lib(P, c, tr)
            items, chosen, info = oracle.generate_policy_best(tr.tensors, ev, tr.n_ops, 0, list(tr.op_phase), limit,
                                                              bpo, sets)
            pol, res, got = P.ss_generate_policy_best(c, ops, tr.tensors, ev, 0, limit, sets)
            assert got == chosen and rows_of(pol) == items and len(items) > 5
            assert (res["peak_with_policy"], res["n_over_with_policy"], res["n_late"], res["bytes"]) == \
                (info["peak"], info["n_over"], info["n_late"], info["bytes"])
        finally:
            P.ss_destroy(c)
