"""Pins for the oracle's trace record and timeline scan (CPU only).

Each test checks the oracle against something other than itself: published
hash vectors, a library routine, the plain live-set definition, brute force
over swap sets, a closed form, or an invariant.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads as W
from workloads.rng import SplitMix64

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- trace record
def test_fnv1a32_published_vectors():
    for line in open(os.path.join(GOLD, "fnv1a32_vectors.txt")):
        if line.startswith("#"):
            continue
        h, _, s = line.rstrip("\n").partition(" ")
        assert oracle.fnv1a32(s.encode()) == int(h, 16)


def record_trace(rec, tr):
    """drive a recorder with a generated trace; returns (ops, events) arrays"""
    rec.begin()
    ev = tr.events
    bounds = np.searchsorted(ev["op_idx"], np.arange(tr.n_ops + 1))
    for i in range(tr.n_ops):
        op = rec.intern(tr.op_name[i], tr.op_stack[i], tr.op_dtype[i],
                        len(tr.op_outputs[i]), tr.op_phase[i])
        rec.record(op, [tuple(e) for e in ev[bounds[i]:bounds[i + 1]].tolist()])
    return rec.ops_array(), rec.events_array()


def test_tokens_dense_first_seen_and_balance():
    tr = W.build_trace(W.config_shape(1))
    rec = oracle.TraceRecorder()
    ops, ev = record_trace(rec, tr)
    # dense ids in first-seen order starting at 1
    first = {}
    for name, tok in zip(tr.op_name, ops["op_token"]):
        first.setdefault(name, int(tok))
    assert sorted(first.values()) == list(range(1, len(first) + 1))
    assert list(first.values()) == sorted(first.values())
    # same name -> same token, same stack -> same hash, and never the padding token
    assert (ops["op_token"] != 0).all()
    for i in range(tr.n_ops):
        assert ops["stack_hash"][i] == oracle.fnv1a32(tr.op_stack[i].encode())
        assert ops["sig"][i] & 0xFF == tr.op_dtype[i]
        assert (ops["sig"][i] >> 16) == tr.op_phase[i]
        assert ops["n_out"][i] == len(tr.op_outputs[i])
    # the recorded events are the generated ones, and an iteration is balanced
    assert np.array_equal(ev, tr.events.astype(ev.dtype))
    assert rec.balance() == 0


def test_recorder_refuses_misplaced_event_and_zero_token():
    rec = oracle.TraceRecorder()
    op = rec.intern("a", "s", 1, 1, 0)
    with pytest.raises(ValueError):
        rec.record(op, [(3, 0, 16)])
    with pytest.raises(ValueError):
        rec.record((0, 1, 1, 1), [])


# -------------------------------------------------------------- timeline scan
def live_set_peak(tensors, away, n_ops, base):
    """Plain definition: P[t] = base + sum of sizes of tensors resident at t.

    A tensor is resident from its alloc operator to its free operator, both
    inclusive, except strictly between t_free and t_in when swapped."""
    P = np.full(n_ops, base, dtype=np.int64)
    for t in tensors:
        tid = int(t["tensor_id"])
        for op in range(int(t["alloc_op"]), int(t["free_op"]) + 1):
            if tid in away and away[tid][0] < op < away[tid][1]:
                continue
            P[op] += int(t["nbytes"])
    return P


def tiny_trace(seed, n_ops=12, T=9):
    rng = SplitMix64(seed, 77)
    tab = np.zeros(T, dtype=W.TENSOR_DT)
    for i in range(T):
        a = rng.randint(n_ops - 4)
        lf = a + rng.randint(2)
        fb = lf + 2 + rng.randint(n_ops - lf - 2)
        fr = min(n_ops - 1, fb + rng.randint(3))
        tab[i] = (i, 1, a, i, a, lf, fb, fr, 0, 0, 256 * (1 + rng.randint(20)))
    from workloads.transformer import events_of
    return tab, events_of(tab)


def policy_events_for(tab, away):
    pe = []
    for tid, (tf, ti) in away.items():
        n = int(tab["nbytes"][tid])
        pe += [(tf, tid, -n), (ti, tid, n)]
    return sorted(pe, key=lambda e: (e[0], e[2] < 0))


def test_late_events_and_amended_records_equal_recording_them_at_once():
    """a hook learns an operator's outputs and its allocations after it recorded the operator: the
    recorder then ends up exactly where recording everything at once would have put it"""
    a, b = oracle.TraceRecorder(), oracle.TraceRecorder()
    with pytest.raises(ValueError):
        a.event(0, 8)                                  # no operator yet
    a.record(a.intern("aten::mm", "s", 1, 2, 0), [(0, 0, 4096), (0, 1, 512)])
    a.record(a.intern("aten::add", "s", 2, 1, 1), [(1, 0, -4096)])
    b.record(b.intern("aten::mm", "s", 0, 0, 0))
    b.event(0, 4096); b.event(1, 512)
    b.amend(0, 1, 2)
    b.record(b.intern("aten::add", "s", 0, 0, 1))
    b.amend(1, 2, 1)
    b.event(0, -4096)
    assert a.ops == b.ops and a.events == b.events and b.balance() == 512
    assert b.ops[1][2] >> 16 == 1                      # the phase survives an amendment


def test_scan_equals_library_cumsum_and_balance():
    tr = W.build_trace(W.config_shape(2))
    base = 12345
    res = oracle.timeline_scan(tr.events, None, tr.n_ops, base, 10**12)
    # generated events are already canonical (operator order, allocs first)
    assert np.array_equal(res["timeline"], base + np.cumsum(tr.events["delta"]))
    assert res["final"] == base                        # alloc/free balance
    assert res["peak"] == max(base, int(res["timeline"].max()))
    # per-operator peak against maximum.accumulate restricted to each operator
    b = np.searchsorted(tr.events["op_idx"], np.arange(tr.n_ops + 1))
    for t in (0, 5, tr.n_ops // 2, tr.n_ops - 1):
        entry = base + int(tr.events["delta"][:b[t]].sum())
        inside = res["timeline"][b[t]:b[t + 1]]
        assert res["per_op"][t] == max([entry] + inside.tolist())


@pytest.mark.parametrize("seed", range(6))
def test_scan_equals_live_set_definition_for_every_swap_subset(seed):
    """brute force over all swap subsets: scan == plain definition, incl. the best subset"""
    tab, ev = tiny_trace(seed)
    n_ops, base = 12, 1000
    cands = [i for i in range(len(tab)) if tab["last_fwd_use"][i] + 1 < tab["first_bwd_use"][i]]
    best_scan, best_def = None, None
    for r in range(len(cands) + 1):
        for sub in itertools.combinations(cands, r):
            away = {i: (int(tab["last_fwd_use"][i]) + 1, int(tab["first_bwd_use"][i])) for i in sub}
            res = oracle.timeline_scan(ev, policy_events_for(tab, away), n_ops, base, 3000)
            P = live_set_peak(tab, away, n_ops, base)
            assert np.array_equal(res["per_op"], P)
            assert res["peak"] == P.max() and res["argpeak_op"] == int(np.argmax(P))
            assert np.array_equal(res["mre"], np.maximum(P - 3000, 0))
            assert res["n_over"] == int((P > 3000).sum())
            assert res["final"] == base
            best_scan = res["peak"] if best_scan is None else min(best_scan, res["peak"])
            best_def = int(P.max()) if best_def is None else min(best_def, int(P.max()))
    assert best_scan == best_def


def test_lifo_staircase_closed_form():
    """tensor i allocated at operator i, freed at operator 2N-1-i: P[t] = base + sum_{i<=min(t,2N-1-t)} s_i"""
    N, base = 7, 50
    s = [3, 1, 4, 1, 5, 9, 2]
    ev = [(i, i, s[i]) for i in range(N)] + [(2 * N - 1 - i, i, -s[i]) for i in range(N)]
    ev.sort(key=lambda e: (e[0], e[2] < 0))
    res = oracle.timeline_scan(ev, None, 2 * N, base, 60)
    for t in range(2 * N):
        assert res["per_op"][t] == base + sum(s[:min(t, 2 * N - 1 - t) + 1])
    assert res["peak"] == base + sum(s) and res["argpeak_op"] == N - 1
    assert res["final"] == base


def test_scan_ignores_event_order_inside_an_operator():
    tab, ev = tiny_trace(3)
    rng = SplitMix64(9)
    ref = oracle.timeline_scan(ev, None, 12, 0, 2000)
    ev2 = ev.copy()
    b = np.searchsorted(ev["op_idx"], np.arange(13))
    for t in range(12):
        seg = ev2[b[t]:b[t + 1]].copy()
        ev2[b[t]:b[t + 1]] = seg[rng.permutation(len(seg))]
    res = oracle.timeline_scan(ev2, None, 12, 0, 2000)
    for key in ("per_op", "mre"):
        assert np.array_equal(ref[key], res[key])
    assert ref["peak"] == res["peak"] and ref["n_over"] == res["n_over"]
    # the running total at the end of every operator does not depend on it either
    ends = b[1:][b[1:] > b[:-1]] - 1
    assert np.array_equal(ref["timeline"][ends], res["timeline"][ends])


def test_swap_free_counts_after_t_free_and_swap_in_before_t_in():
    # one tensor of 100 bytes alive over operators 0..9, away strictly between 3 and 7
    ev = [(0, 0, 100), (9, 0, -100)]
    pe = [(3, 0, -100), (7, 0, 100)]
    res = oracle.timeline_scan(ev, pe, 10, 0, 50)
    assert res["per_op"].tolist() == [100, 100, 100, 100, 0, 0, 0, 100, 100, 100]
    assert res["n_over"] == 7 and res["mre"][0] == 50


def test_scan_rejects_event_beyond_last_operator():
    with pytest.raises(ValueError):
        oracle.timeline_scan([(5, 0, 1)], None, 5, 0, 0)


def test_empty_trace():
    res = oracle.timeline_scan([], None, 0, 7, 0)
    assert res["peak"] == 7 and res["argpeak_op"] == -1 and len(res["timeline"]) == 0
    res = oracle.timeline_scan([], None, 3, 7, 5)
    assert res["per_op"].tolist() == [7, 7, 7] and res["n_over"] == 3
