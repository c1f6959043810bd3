"""The library at the boundary cases of tests/test_oracle_boundaries.py (hand-worked there): the same
inputs through the C ABI, compared with the oracle and with the hand-worked values."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import assert_applied_equal
from test_oracle_trace_timeline import live_set_peak
from test_oracle_generator import table
from test_oracle_boundaries import abc, rows_for, spike_case, BIG
from test_gpu_generator import make_ctx, ops_with_phases, rows_of, check_against_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2509_11076_amd.binding as B
    return B


def test_scan_canonical_order_and_one_byte_excess(P):
    c = make_ctx(P, staging_bytes=4096)
    try:
        ev = np.array([(0, 1, 100), (1, 2, -20), (1, 3, 30), (2, 1, -80)], dtype=W.EVENT_DT)   # release listed first
        pe = np.array([(1, 8, 50), (1, 9, -10)], dtype=W.EVENT_DT)
        lib = P.ss_timeline_scan(c, ev, pe, 3, 7, 156, want_timeline=True)
        assert lib["timeline"].tolist() == [107, 157, 187, 167, 157, 77]
        assert lib["per_op"].tolist() == [107, 187, 157] and lib["mre"].tolist() == [0, 31, 1]
        assert lib["n_over"] == 2 and lib["argpeak_op"] == 1 and lib["final"] == 77
    finally:
        P.ss_destroy(c)


def apply_both(P, pol, idx, tab, bpo, flags=0, keep=False, points=False):
    ora = oracle.apply_policy(pol, idx, tab, bpo, keep_late=keep, policy_points=points)
    c = make_ctx(P, staging_bytes=max(4096, ora["staging_bytes"]), link_bytes_per_op=bpo,
                 flags=flags | (P.SS_CFG_KEEP_LATE if keep else 0) | (P.SS_CFG_POLICY_POINTS if points else 0))
    try:
        lib = P.ss_apply_policy(c, pol, np.asarray(idx, dtype=np.int64), tab)      # unbound: computed, not loaded
        o = dict(ora)
        assert_applied_equal(dict(lib, n_kept=0), P, c, o)                          # arrays; no schedule to view
        return lib, ora
    finally:
        P.ss_destroy(c)


def test_apply_hand_cases(P):
    tab = abc()
    lib, ora = apply_both(P, rows_for(tab), [0, 1, 2], tab, BIG)
    assert [tuple(r)[4:8] for r in lib["resolved"].tolist()] == [(2, 3, 9, 10), (2, 3, 8, 9), (3, 4, 8, 9)]
    assert lib["n_out_batches"] == 2 and lib["n_in_batches"] == 2 and lib["staging_bytes"] == 6144
    assert {(a[1], a[2]): a[3] for a in lib["actions"].tolist()} == {(a[1], a[2]): a[3] for a in ora["actions"]}
    # the tensor grew since the policy was made
    pol = rows_for(tab)
    pol["nbytes"][1] = 1999
    lib, _ = apply_both(P, pol, [0, 1, 2], tab, BIG)
    assert [int(f) & P.SS_F_RESIZED for f in lib["resolved"]["flags"]] == [0, P.SS_F_RESIZED, 0]
    # points on the uses themselves are kept, release point == swap-in point is not
    pts = rows_for(tab)
    for a, (tf, ti) in enumerate([(2, 10), (5, 5), (3, 9)]):
        t = tab[a]
        pts[a] = (int(t["producer_op"]), 0, a, 0, int(t["last_fwd_use"]), tf, ti, int(t["first_bwd_use"]), int(t["nbytes"]))
    lib, _ = apply_both(P, pts, [0, 1, 2], tab, BIG, points=True)
    assert [bool(int(f) & P.SS_F_ORDER) for f in lib["resolved"]["flags"]] == [False, True, False]
    # swap-in floor, slot rounding
    tab2 = table([(0, 1, 7, 8, 257), (1, 5, 9, 10, 1)])
    lib, _ = apply_both(P, rows_for(tab2), [0, 1], tab2, BIG)
    assert [tuple(r)[3:8] for r in lib["resolved"].tolist()] == [(0, 1, 2, 6, 7), (0, 5, 6, 8, 9)]
    assert lib["descs_out"]["host_off"].tolist() == [0, 512] and lib["staging_bytes"] == 768
    # an allocation before a release of the same operator
    tab3 = table([(0, 2, 8, 9, 100), (1, 6, 10, 11, 200)])
    pts = rows_for(tab3)
    pts[0] = (0, 0, 0, 0, 2, 5, 7, 8, 100)
    pts[1] = (1, 0, 1, 0, 6, 7, 9, 10, 200)
    lib, _ = apply_both(P, pts, [0, 1], tab3, BIG, points=True)
    assert [tuple(e) for e in lib["policy_events"].tolist()] == [(5, 0, -100), (7, 0, 100), (7, 1, -200), (9, 1, 200)]
    # tensors with a use missing, or no room between their uses
    tab4 = table([(0, 2, W.NONE_OP, 5, 100), (1, W.NONE_OP, 4, 5, 100), (2, 2, 5, 5, 100), (3, 3, 3, 5, 100), (4, 3, 4, 5, 100)])
    lib, _ = apply_both(P, rows_for(tab4), [0, 1, 2, 3, 4], tab4, BIG)
    assert [bool(int(f) & P.SS_F_ORDER) for f in lib["resolved"]["flags"]] == [True, True, False, True, True]
    # release point at an exact operator boundary: 100 link bytes per operator, 100 and 101 bytes
    for n, want in ((100, (0, 1, 4, 5)), (101, (0, 2, 3, 5))):     # 101 bytes spill into a second operator, both ways
        tab5 = table([(0, 0, 5, 6, n)])
        lib, _ = apply_both(P, rows_for(tab5), [0], tab5, 100)
        assert tuple(lib["resolved"].tolist()[0])[4:8] == want


def test_match_landings_on_operator_zero(P):
    c = make_ctx(P, staging_bytes=4096)
    try:
        ops = np.array([(1, 7, 0x101, 1), (2, 7, 0x101, 1), (3, 7, 0x101, 2)], dtype=W.OP_DT)
        anc = np.array([(0, 0), (2, 1), (3, 0), (2, 2)], dtype=W.ANCHOR_DT)
        m = P.ss_match_sequence(c, ops, ops, anc)
        assert m["new_idx"].tolist() == [0, 2, -1, -1] and m["level"].tolist() == [0, 0, 255, 255] and m["n_unmatched"] == 2
        m = P.ss_match_sequence(c, ops, ops, anc, flags=P.SS_MATCH_ALIGN)
        assert m["new_idx"].tolist() == [0, 2, -1, -1] and m["n_unmatched"] == 2
    finally:
        P.ss_destroy(c)


def gen(P, tab, phases, limit, bpo, g=64, per_phase=None, **kw):
    ev = W.transformer.events_of(tab)
    c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo)
    try:
        return check_against_oracle(P, c, ops_with_phases(phases), phases, tab, ev, len(phases), limit, bpo, g, g,
                                    per_phase=per_phase, **kw)
    finally:
        P.ss_destroy(c)


def test_generator_boundaries(P):
    # reach of a tensor: strictly after the operator following its last forward use, before the swap-in layer
    for p, want in ((3, None), (4, [(0, 0, 0, 0, 2, 3, 11, 12, 300)]), (10, [(0, 0, 0, 0, 2, 3, 11, 12, 300)]), (11, None), (12, None)):
        tab, mem, phases, limit = spike_case(p)
        assert gen(P, tab, phases, limit, BIG) == want
    # strictly more time than the transfer takes, in either direction
    tab, mem, phases, limit = spike_case(6)
    assert gen(P, tab, phases, limit, 300) == [(0, 0, 0, oracle.F_LATE, 2, 10, 11, 12, 300)]
    assert gen(P, tab, phases, limit, 301) == [(0, 0, 0, 0, 2, 3, 11, 12, 300)]
    assert gen(P, tab, phases, limit, 1000, per_phase=(300, 301, 301)) == [(0, 0, 0, 0, 2, 8, 11, 12, 300)]
    assert gen(P, tab, phases, limit, 1000, per_phase=(301, 300, 300)) == [(0, 0, 0, 0, 2, 3, 7, 12, 300)]
    # minimum size inclusive
    assert len(gen(P, tab, phases, limit, BIG, min_bytes=300)) == 1
    assert gen(P, tab, phases, limit, BIG, min_bytes=301) is None
    # every layer visited on the way down
    tab = table([(0, 2, 12, 13, 300), (1, 2, 12, 13, 300), (6, 6, W.NONE_OP, 6, 500)])
    assert gen(P, tab, [0] * 8 + [1] * 8, 650, 301) == [(0, 0, 0, 0, 2, 3, 11, 12, 300), (1, 0, 1, 0, 2, 4, 10, 12, 300)]
    # fallback layer between neighbouring layers
    tab = table([(0, 1, 6, 7, 300), (3, 3, W.NONE_OP, 3, 200)])
    assert gen(P, tab, [0] * 4 + [1] * 4, 400, 10, g=1) == [(0, 0, 0, oracle.F_LATE, 1, 3, 4, 6, 300)]
    # Eq. 2: normalised by the largest size; the count taken strictly inside the idle span
    phases = [0] * 12 + [1] * 12
    tab = table([(0, 0, 23, 23, 100), (0, 12, 15, 16, 300), (5, 5, W.NONE_OP, 14, 500)])
    assert [it[2] for it in gen(P, tab, phases, 850, BIG)] == [0]
    for size_u, size_v in ((100, 200), (200, 100)):
        tab = table([(0, 0, 23, 23, 50), (0, 0, 14, 15, size_u), (0, 4, 23, 23, size_v), (5, 5, W.NONE_OP, 14, 500)])
        mem = live_set_peak(tab, {}, 24, 0)
        gen(P, tab, phases, int(mem.max()) - 40, BIG, c_num=0, c_den=1)
