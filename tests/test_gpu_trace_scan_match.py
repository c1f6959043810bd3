"""GPU parity: trace record, timeline scan, sequence match, policy application and greedy
policy of the HIP library against the CPU oracle, element by element (exact equality:
everything is integers).  All calls go through the C ABI."""
import os

import numpy as np
import pytest

import oracle
import workloads as W
from workloads.arena import place_tensors
from workloads.rng import SplitMix64
from helpers import record_oracle, record_lib, ops_tuples, assert_applied_equal
from test_oracle_trace_timeline import tiny_trace, policy_events_for

pytestmark = pytest.mark.gpu
INSTANT = 1 << 40
PERT = dict(p_drop=0.1, p_insert=0.1, moe_max=8, seq_jitter=0.15)


@pytest.fixture(scope="module")
def P():
    import paper_2509_11076_amd.binding as B
    return B


@pytest.fixture()
def ctx(P):
    cfg = P.ss_config_default()
    cfg.staging_bytes = 1 << 20
    cfg.max_ops = 1 << 16
    cfg.max_events = 1 << 18
    c = P.ss_create(cfg)
    yield c
    P.ss_destroy(c)


def make_ctx(P, **kw):
    cfg = P.ss_config_default()
    for k, v in kw.items():
        setattr(cfg, k, v)
    return P.ss_create(cfg)


# ------------------------------------------------------------------ trace record
@pytest.mark.parametrize("cfgno", [1, 2])
def test_trace_record_is_byte_identical(P, ctx, cfgno):
    tr = W.build_trace(W.config_shape(cfgno))
    o_ops, o_ev = record_oracle(oracle.TraceRecorder(), tr)
    l_ops, l_ev, bal = record_lib(P, ctx, tr)
    assert np.array_equal(l_ops.view(np.uint8), o_ops.view(np.uint8))
    assert np.array_equal(l_ev.view(np.uint8), o_ev.view(np.uint8))
    assert bal == 0


def test_trace_tokens_persist_across_iterations_and_errors(P, ctx):
    rec = oracle.TraceRecorder()
    shape = W.ModelShape("naive", 64, 3, 4, 64, 1, 4, experts0=4)
    for it in range(3):
        tr = W.build_trace(shape, iteration=it, perturb=PERT if it else None)
        o_ops, o_ev = record_oracle(rec, tr)
        l_ops, l_ev, bal = record_lib(P, ctx, tr)
        assert np.array_equal(l_ops.view(np.uint8), o_ops.view(np.uint8))
        assert np.array_equal(l_ev.view(np.uint8), o_ev.view(np.uint8)) and bal == 0
    P.ss_trace_begin(ctx)
    op = P.ss_intern_op(ctx, "x", "y", 1, 1, 0)
    bad = np.zeros(1, P.EVENT_DT); bad["op_idx"] = 5; bad["delta"] = 8
    with pytest.raises(P.SsError) as e:
        P.ss_trace_record(ctx, op, bad)
    assert e.value.code == P.SS_E_INVAL
    zero = op.copy(); zero["op_token"] = 0
    with pytest.raises(P.SsError):
        P.ss_trace_record(ctx, zero)
    # events and output counts that arrive after the operator was recorded (dispatch hooks)
    rec2 = oracle.TraceRecorder()
    P.ss_trace_begin(ctx)
    with pytest.raises(P.SsError) as e:
        P.ss_trace_event(ctx, 0, 8)
    assert e.value.code == P.SS_E_ORDER
    for i, (nm, ph) in enumerate((("x", 0), ("z", 1), ("x", 2))):
        P.ss_trace_record(ctx, P.ss_intern_op(ctx, nm, "y", 0, 0, ph))
        rec2.record(rec2.intern(nm, "y", 0, 0, ph))
        for tid, d in ((3 * i, 4096), (3 * i + 1, -512)):
            P.ss_trace_event(ctx, tid, d)
            rec2.event(tid, d)
        P.ss_trace_amend(ctx, i, 4 + i, i + 1)
        rec2.amend(i, 4 + i, i + 1)
    l_ops, l_ev, bal = P.ss_trace_view(ctx)
    assert np.array_equal(l_ops["sig"], rec2.ops_array()["sig"]) and np.array_equal(l_ops["n_out"], rec2.ops_array()["n_out"])
    assert np.array_equal(l_ev.view(np.uint8), rec2.events_array().view(np.uint8)) and bal == rec2.balance()
    with pytest.raises(P.SsError) as e:
        P.ss_trace_amend(ctx, 3, 1, 1)
    assert e.value.code == P.SS_E_INVAL
    small = make_ctx(P, staging_bytes=4096, max_ops=2, max_events=4)
    try:
        P.ss_trace_record(small, op); P.ss_trace_record(small, op)
        with pytest.raises(P.SsError) as e:
            P.ss_trace_record(small, op)
        assert e.value.code == P.SS_E_CAPACITY
    finally:
        P.ss_destroy(small)


# ------------------------------------------------------------------ timeline scan
def assert_scan_equal(lib, ora, timeline=True):
    assert lib["peak"] == ora["peak"] and lib["argpeak_op"] == ora["argpeak_op"]
    assert lib["n_over"] == ora["n_over"] and lib["final"] == ora["final"]
    assert np.array_equal(lib["per_op"], ora["per_op"]) and np.array_equal(lib["mre"], ora["mre"])
    if timeline:
        assert np.array_equal(lib["timeline"], ora["timeline"])


@pytest.mark.parametrize("seed", range(4))
def test_scan_tiny_traces_with_policy_events(P, ctx, seed):
    tab, ev = tiny_trace(seed)
    away = {i: (int(tab["last_fwd_use"][i]) + 1, int(tab["first_bwd_use"][i]))
            for i in range(len(tab)) if i % 2 == seed % 2 and tab["last_fwd_use"][i] + 1 < tab["first_bwd_use"][i]}
    pe = policy_events_for(tab, away)
    pe_arr = np.array(pe, dtype=W.EVENT_DT) if pe else None
    ora = oracle.timeline_scan(ev, pe, 12, 1000, 3000)
    lib = P.ss_timeline_scan(ctx, ev, pe_arr, 12, 1000, 3000, want_timeline=True)
    assert_scan_equal(lib, ora)


@pytest.mark.parametrize("cfgno,budget", [(1, 2 << 20), (2, 4 << 30), (3, 48 * 10**9)])
def test_scan_transformer_traces(P, ctx, cfgno, budget):
    tr = W.build_trace(W.config_shape(cfgno))
    ora = oracle.timeline_scan(tr.events, None, tr.n_ops, 7 << 30, budget)
    lib = P.ss_timeline_scan(ctx, tr.events, None, tr.n_ops, 7 << 30, budget, want_timeline=True)
    assert_scan_equal(lib, ora)
    assert lib["sorted"] == 1


def test_scan_stress_trace_100k_events_spanning_many_chunks(P):
    tr, pol, _ = W.build_small_tensor_stress()
    assert len(tr.events) == 100000
    c = make_ctx(P, staging_bytes=4096)
    try:
        budget = 6 * 10**9
        ora = oracle.timeline_scan(tr.events, None, tr.n_ops, 0, budget)
        lib = P.ss_timeline_scan(c, tr.events, None, tr.n_ops, 0, budget, want_timeline=True)
        assert_scan_equal(lib, ora)
        # with the policy events of the whole swap set (40,000 more events)
        ap = oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, 256 << 20)
        pe = np.array(ap["policy_events"], dtype=W.EVENT_DT)
        ora = oracle.timeline_scan(tr.events, pe, tr.n_ops, 0, budget)
        lib = P.ss_timeline_scan(c, tr.events, pe, tr.n_ops, 0, budget, want_timeline=True)
        assert_scan_equal(lib, ora)
    finally:
        P.ss_destroy(c)


def test_scan_batch_of_candidate_policies_in_one_launch(P, ctx):
    """many candidate policies against one trace: every scan of the batch equals the oracle's scan of
    that candidate alone"""
    tr = W.build_trace(W.config_shape(2))
    tab = tr.tensors
    keep = np.nonzero((tab["first_bwd_use"] != W.NONE_OP) & (tab["last_fwd_use"] != W.NONE_OP)
                      & (tab["last_fwd_use"] + 1 < tab["first_bwd_use"]))[0]
    rng = SplitMix64(4, 9)
    cands = []
    for c in range(19):
        away = {}
        for row in keep:
            if rng.randint(19) < c:                   # candidate c swaps about c/19 of the tensors
                lf, fb = int(tab["last_fwd_use"][row]), int(tab["first_bwd_use"][row])
                tf = lf + rng.randint(fb - lf)
                away[int(tab["tensor_id"][row])] = (tf, tf + 1 + rng.randint(fb - tf))
        pe = policy_events_for(tab, away)
        a = np.zeros(len(pe), dtype=W.EVENT_DT)
        for i, e in enumerate(pe):
            a[i] = e
        cands.append(a)
    no = oracle.timeline_scan(tr.events, None, tr.n_ops, 7, 0)
    budget = int(no["peak"] * 0.7)
    lib = P.ss_timeline_scan_batch(ctx, tr.events, cands, tr.n_ops, 7, budget, want_per_op=True)
    assert len(lib) == 19
    peaks = []
    for c, a in enumerate(cands):
        ora = oracle.timeline_scan(tr.events, a, tr.n_ops, 7, budget)
        assert (lib[c]["peak"], lib[c]["argpeak_op"], lib[c]["n_over"], lib[c]["final"]) == \
            (ora["peak"], ora["argpeak_op"], ora["n_over"], ora["final"]), c
        assert np.array_equal(lib[c]["per_op"], ora["per_op"])
        peaks.append(ora["peak"])
    assert lib[0]["peak"] == no["peak"] and min(peaks) < 0.8 * no["peak"] and len(set(peaks)) > 10
    # tiny traces, empty candidate lists, no candidates, an operator out of range in one candidate
    tab, ev = tiny_trace(3)
    one = P.ss_timeline_scan_batch(ctx, ev, [None, None], 12, 0, 1 << 40)
    assert one[0]["peak"] == one[1]["peak"] == oracle.timeline_scan(ev, None, 12, 0, 1 << 40)["peak"]
    assert P.ss_timeline_scan_batch(ctx, ev, [], 12, 0, 0) == []
    bad = np.zeros(1, dtype=W.EVENT_DT); bad[0] = (12, 0, 8)
    with pytest.raises(P.SsError) as e:
        P.ss_timeline_scan_batch(ctx, ev, [None, bad], 12, 0, 0)
    assert e.value.code == P.SS_E_INVAL


def test_scan_unsorted_events_edge_cases(P, ctx):
    tab, ev = tiny_trace(5)
    perm = SplitMix64(4).permutation(len(ev))
    shuffled = ev[perm]
    ora = oracle.timeline_scan(ev, None, 12, 0, 2500)
    lib = P.ss_timeline_scan(ctx, shuffled, None, 12, 0, 2500)          # any order: per-operator results hold
    assert_scan_equal(lib, ora, timeline=False)
    assert lib["sorted"] == 0
    with pytest.raises(P.SsError) as e:                                 # the timeline needs operator order
        P.ss_timeline_scan(ctx, shuffled, None, 12, 0, 2500, want_timeline=True)
    assert e.value.code == P.SS_E_ORDER
    with pytest.raises(P.SsError) as e:                                 # event beyond the last operator
        P.ss_timeline_scan(ctx, ev, None, 5, 0, 0)
    assert e.value.code == P.SS_E_INVAL
    # no events, no operators
    lib = P.ss_timeline_scan(ctx, None, None, 0, 7, 0, want_timeline=True)
    assert lib["peak"] == 7 and lib["argpeak_op"] == -1 and lib["final"] == 7
    lib = P.ss_timeline_scan(ctx, None, None, 3, 7, 5)
    assert lib["per_op"].tolist() == [7, 7, 7] and lib["n_over"] == 3 and lib["argpeak_op"] == 0
    # more operators than one pass of the workgroup covers, large values
    n_ops = 5000
    big = np.zeros(2 * n_ops, dtype=W.EVENT_DT)
    big["op_idx"] = np.repeat(np.arange(n_ops), 2)
    big["delta"][0::2] = (np.arange(n_ops) % 97 + 1) * (1 << 33)
    big["delta"][1::2] = -((np.arange(n_ops) % 89 + 1) * (1 << 32))
    ora = oracle.timeline_scan(big, None, n_ops, -5, 1 << 40)
    lib = P.ss_timeline_scan(ctx, big, None, n_ops, -5, 1 << 40, want_timeline=True)
    assert_scan_equal(lib, ora)


# ------------------------------------------------------------------ sequence match
def traces_for_match(it, shape=None, rec=None):
    shape = shape or W.ModelShape("naive", 64, 6, 4, 64, 1, 4, experts0=4)
    tr0 = W.build_trace(shape, iteration=0)
    tr1 = W.build_trace(shape, iteration=it, perturb=PERT)
    rec = rec or oracle.TraceRecorder()
    ref, _ = record_oracle(rec, tr0)
    cur, _ = record_oracle(rec, tr1)
    tab = tr0.tensors
    keep = (tab["first_bwd_use"] != W.NONE_OP) & (tab["last_fwd_use"] != W.NONE_OP)
    anchors = np.zeros(int(keep.sum()), dtype=W.ANCHOR_DT)
    anchors["ref_op"] = tab["producer_op"][keep]; anchors["out_slot"] = tab["out_slot"][keep]
    return ref, cur, anchors, tr0, tr1


@pytest.mark.parametrize("it", [1, 2, 3])
def test_match_perturbed_sequences(P, ctx, it):
    ref, cur, anchors, _, _ = traces_for_match(it)
    ora = oracle.match_sequence(ops_tuples(ref), ops_tuples(cur), anchors.tolist())
    lib = P.ss_match_sequence(ctx, ref, cur, anchors)
    assert (lib["dot"], lib["na"], lib["nb"], lib["similar"]) == (ora["dot"], ora["na"], ora["nb"], ora["similar"])
    assert np.array_equal(lib["new_idx"], ora["new_idx"]) and np.array_equal(lib["level"], ora["level"])
    assert lib["n_unmatched"] == ora["n_unmatched"]
    # histogram reading of the cosine
    ora_h = oracle.similarity(cur["op_token"], ref["op_token"], histogram=True)
    lib_h = P.ss_match_sequence(ctx, ref, cur, None, flags=P.SS_MATCH_HISTOGRAM)
    assert (lib_h["similar"], lib_h["dot"], lib_h["na"], lib_h["nb"]) == ora_h


@pytest.mark.parametrize("flags_name", ["keyed", "aligned"])
def test_match_of_a_sequence_with_itself_and_with_one_operator_changed(P, ctx, flags_name):
    """the current sequence being the reference itself is answered on the host without the kernels; the
    result is the oracle's all the same (anchors beyond the sequence, on output slots the operator does not
    have, several on one place), and so is the kernels' answer once a single operator differs"""
    ref, _, anchors, tr0, _ = traces_for_match(1)
    n = len(ref)
    extra = np.zeros(7, dtype=W.ANCHOR_DT)
    extra[0] = (n + 3, 0)                                  # beyond the sequence
    extra[1] = (int(anchors["ref_op"][0]), 200)            # a slot no operator has
    extra[2] = anchors[4]; extra[3] = anchors[4]           # one place, three claimants with anchors[4] itself
    extra[4] = (0, 0); extra[5] = (n - 1, 0); extra[6] = (n - 1, 1)
    anc = np.concatenate([anchors, extra])
    flags = P.SS_MATCH_ALIGN if flags_name == "aligned" else 0

    def both(cur):
        lib = P.ss_match_sequence(ctx, ref, cur, anc, flags=flags)
        ora = oracle.match_sequence(ops_tuples(ref), ops_tuples(cur), anc.tolist())
        if flags:
            al = oracle.align_anchors(ops_tuples(ref), ops_tuples(cur), anc.tolist())
            ora = dict(ora, new_idx=al["new_idx"], level=al["level"], n_unmatched=int((al["new_idx"] < 0).sum()))
        assert np.array_equal(lib["new_idx"], ora["new_idx"]) and np.array_equal(lib["level"], ora["level"])
        assert (lib["dot"], lib["na"], lib["nb"], lib["similar"], lib["n_unmatched"]) == \
            (ora["dot"], ora["na"], ora["nb"], ora["similar"], ora["n_unmatched"])
        return lib
    same = both(ref.copy())
    assert same["similar"] and same["dot"] == same["na"] == same["nb"]
    assert (same["new_idx"][:len(anchors)] == anchors["ref_op"]).all()
    cur = ref.copy()
    cur["stack_hash"][n // 2] ^= 0x5A5A                    # one operator reached by another call path
    near = both(cur)
    assert near["similar"] and near["dot"] == same["dot"]


def test_match_full_7b_shape_varying_sequence(P, ctx):
    ref, cur, anchors, tr0, tr1 = traces_for_match(2, W.config_shape(4))
    assert len(ref) > 1000 and len(anchors) > 400
    ora = oracle.match_sequence(ops_tuples(ref), ops_tuples(cur), anchors.tolist())
    lib = P.ss_match_sequence(ctx, ref, cur, anchors)
    assert np.array_equal(lib["new_idx"], ora["new_idx"]) and np.array_equal(lib["level"], ora["level"])
    assert (lib["dot"], lib["na"], lib["nb"], lib["similar"]) == (ora["dot"], ora["na"], ora["nb"], ora["similar"])
    # identical sequence: every anchor stays, level 0, similar
    lib = P.ss_match_sequence(ctx, ref, ref, anchors)
    assert np.array_equal(lib["new_idx"], anchors["ref_op"].astype(np.int32)) and (lib["level"] == 0).all()
    assert lib["similar"] and lib["dot"] == lib["na"] == lib["nb"]


def test_match_threshold_stage_machine_and_edges(P, ctx):
    def seq(tokens):
        a = np.zeros(len(tokens), dtype=W.OP_DT)
        a["op_token"] = tokens; a["n_out"] = 1
        return a
    # exact 19/20 cosine is not similar; just above is (comparator in exact integers)
    r = P.ss_match_sequence(ctx, seq([19, 5, 3, 2, 1]), seq([1, 0, 0, 0, 0]), None)
    assert (r["dot"], r["na"], r["nb"], r["similar"]) == (19, 1, 400, False)
    r = P.ss_match_sequence(ctx, seq([20, 5, 3, 2, 1]), seq([1, 0, 0, 0, 0]), None)
    assert (r["dot"], r["na"], r["nb"], r["similar"]) == (20, 1, 439, True)
    # length test, relative to the reference, strict
    assert P.ss_match_sequence(ctx, seq([1] * 100), seq([1] * 104), None)["similar"]
    assert not P.ss_match_sequence(ctx, seq([1] * 100), seq([1] * 105), None)["similar"]
    assert P.ss_match_sequence(ctx, seq([]), seq([]), None)["similar"]
    assert not P.ss_match_sequence(ctx, seq([]), seq([1]), None)["similar"]
    # sums near the documented limit: 2^17-sized tokens, 2^16 operators
    big = seq([(1 << 17) + (i % 7) for i in range(1 << 16)])
    o = oracle.similarity(big["op_token"], big["op_token"])
    r = P.ss_match_sequence(ctx, big, big, None)
    assert (r["similar"], r["dot"], r["na"], r["nb"]) == o
    with pytest.raises(P.SsError):                          # token beyond 2^18
        P.ss_match_sequence(ctx, seq([1 << 18]), seq([1]), None)
    # stage machine against the hand-derived table (Algo. 1, m = 2, n = 5)
    gold = os.path.join(os.path.dirname(__file__), "golden", "stage_machine_m2_n5.txt")
    names = {"WarmUp": P.SS_STAGE_WARMUP, "GenPolicy": P.SS_STAGE_GENPOLICY, "Stable": P.SS_STAGE_STABLE}
    cases = {}
    for line in open(gold):
        if line.startswith("#") or not line.strip():
            continue
        c, it, sim, step, stage = line.split()
        cases.setdefault(c, []).append((int(sim), int(step), names[stage]))
    same, other = seq([3, 1, 4, 1, 5]), seq([9, 9, 9, 9, 9, 9, 9, 9, 9])
    for c in sorted(cases):
        fresh = make_ctx(P, staging_bytes=4096)
        try:
            for sim, step, stage in cases[c]:
                r = P.ss_match_sequence(fresh, same, same if sim else other, None, flags=P.SS_MATCH_STEP_STAGE)
                assert r["similar"] == bool(sim) and r["stage"] == stage and r["stable_step"] == step
        finally:
            P.ss_destroy(fresh)


def test_match_relaxation_and_injectivity_cases(P, ctx):
    def ops(rows):
        return np.array(rows, dtype=W.OP_DT)
    ref = ops([(1, 10, 0x101, 1), (1, 10, 0x101, 1), (2, 20, 0x201, 2)])
    cur = ops([(1, 11, 0x101, 1), (1, 12, 0x10101, 1), (2, 20, 0x202, 2)])
    anc = np.array([(0, 0), (1, 0), (2, 1), (2, 5), (7, 0)], dtype=W.ANCHOR_DT)
    o_idx, o_lvl = oracle.match_anchors(ops_tuples(ref), ops_tuples(cur), anc.tolist())
    r = P.ss_match_sequence(ctx, ref, cur, anc)
    assert r["new_idx"].tolist() == o_idx.tolist() == [0, 1, -1, -1, -1]
    assert r["level"].tolist() == o_lvl.tolist()
    ref = ops([(1, 1, 1, 1), (1, 2, 1, 1)]); cur = ops([(1, 3, 1, 1)])
    anc = np.array([(0, 0), (1, 0), (0, 0)], dtype=W.ANCHOR_DT)
    r = P.ss_match_sequence(ctx, ref, cur, anc)
    assert r["new_idx"].tolist() == [0, -1, -1] and r["n_unmatched"] == 2
    # sequences longer than one wavefront strip, anchor at the very end
    n = 300
    ref = ops([(1 + i % 3, 7, 0x101, 1) for i in range(n)])
    cur = ops([(9, 9, 0x101, 1)] * 70 + [(1 + i % 3, 7, 0x101, 1) for i in range(n)])
    anc = np.array([(n - 1, 0), (0, 0), (64, 0), (63, 0)], dtype=W.ANCHOR_DT)
    o_idx, o_lvl = oracle.match_anchors(ops_tuples(ref), ops_tuples(cur), anc.tolist())
    r = P.ss_match_sequence(ctx, ref, cur, anc)
    assert r["new_idx"].tolist() == o_idx.tolist() == [n - 1 + 70, 70, 134, 133]


def test_match_many_anchors_on_few_landings(P, ctx):
    """thousands of anchors drawn (with repetition) from a few hundred (operator, slot) pairs, some
    of them beyond the operator's outputs or beyond the sequence: for every landing the lowest
    anchor index keeps it, all later ones lose it"""
    rng = SplitMix64(21, 4)
    n = 700
    ops = np.zeros(n, dtype=W.OP_DT)
    ops["op_token"] = [1 + rng.randint(40) for _ in range(n)]
    ops["stack_hash"] = [rng.randint(3) for _ in range(n)]
    ops["sig"] = 0x0101
    ops["n_out"] = [1 + rng.randint(3) for _ in range(n)]
    cur = np.concatenate([ops[:200], ops[230:]])                      # thirty operators missing
    k = 6000
    anc = np.zeros(k, dtype=W.ANCHOR_DT)
    anc["ref_op"] = [rng.randint(n + 5) if rng.randint(8) == 0 else rng.randint(60) * 11 for _ in range(k)]
    anc["out_slot"] = [rng.randint(4) for _ in range(k)]
    o_idx, o_lvl = oracle.match_anchors(ops_tuples(ops), ops_tuples(cur), anc.tolist())
    r = P.ss_match_sequence(ctx, ops, cur, anc)
    assert np.array_equal(r["new_idx"], o_idx) and np.array_equal(r["level"], o_lvl)
    assert r["n_unmatched"] == int((o_idx < 0).sum()) > k // 2
    kept = r["new_idx"] >= 0
    assert 100 < kept.sum() < 1000
    pairs = set(zip(r["new_idx"][kept].tolist(), anc["out_slot"][kept].tolist()))
    assert len(pairs) == kept.sum()                                   # injective


def test_scan_long_runs_of_one_operator_sorted_and_not(P, ctx):
    """runs of one operator's events far longer than a wavefront and a workgroup pass, runs of length
    one, operators without events; once in operator order, once with whole runs moved out of order"""
    rng = SplitMix64(33, 2)
    n_ops = 300
    runs = []
    for t in range(n_ops):
        length = [0, 1, 2, 63, 64, 65, 130, 1500, 2300][rng.randint(9)]
        ev = np.zeros(length, dtype=W.EVENT_DT)
        ev["op_idx"] = t
        ev["tensor_id"] = np.arange(length)
        ev["delta"] = [(1 + rng.randint(1 << 20)) * (1 if rng.randint(3) else -1) for _ in range(length)]
        runs.append(ev)
    ev = np.concatenate(runs)
    assert len(ev) > 100000
    pe = np.zeros(4000, dtype=W.EVENT_DT)
    pe["op_idx"] = np.sort(np.array([rng.randint(n_ops) for _ in range(4000)]))
    pe["delta"] = [(1 + rng.randint(1 << 22)) * (1 if rng.randint(2) else -1) for _ in range(4000)]
    ora = oracle.timeline_scan(ev, pe, n_ops, 11, 1 << 28)
    lib = P.ss_timeline_scan(ctx, ev, pe, n_ops, 11, 1 << 28, want_timeline=True)
    assert_scan_equal(lib, ora)
    order = SplitMix64(5).permutation(n_ops)
    moved = np.concatenate([runs[i] for i in order])
    lib = P.ss_timeline_scan(ctx, moved, pe, n_ops, 11, 1 << 28)
    assert_scan_equal(lib, ora, timeline=False)
    assert lib["sorted"] == 0
    # at this length the gather runs in many workgroups: their flags must come together as in one
    with pytest.raises(P.SsError) as e:
        P.ss_timeline_scan(ctx, moved, pe, n_ops, 11, 1 << 28, want_timeline=True)
    assert e.value.code == P.SS_E_ORDER
    bad = ev.copy()
    bad["op_idx"][len(bad) - 7] = n_ops                                 # one event beyond the last operator, far into the list
    with pytest.raises(P.SsError) as e:
        P.ss_timeline_scan(ctx, bad, pe, n_ops, 11, 1 << 28)
    assert e.value.code == P.SS_E_INVAL
    bad_pe = pe.copy()
    bad_pe["op_idx"][-1] = n_ops + 5
    with pytest.raises(P.SsError) as e:
        P.ss_timeline_scan(ctx, ev, bad_pe, n_ops, 11, 1 << 28)
    assert e.value.code == P.SS_E_INVAL
    again = P.ss_timeline_scan(ctx, ev, pe, n_ops, 11, 1 << 28, want_timeline=True)       # and nothing is left behind
    assert_scan_equal(again, ora)


# ------------------------------------------------------------------ apply policy / greedy
@pytest.mark.parametrize("cfgno,bpo,guard", [(1, 64 * 1024, 256), (1, INSTANT, 0), (1, 16, 0),
                                             (2, 8 << 20, 0), (2, 64 << 20, 512)])
def test_apply_policy_prescribed_sets(P, cfgno, bpo, guard):
    import torch
    tr = W.build_trace(W.config_shape(cfgno))
    pol = W.config_swap_set(tr, cfgno)
    arena_bytes = place_tensors(tr.tensors, guard=guard)
    idx = pol["ref_op"].astype(np.int64)
    idx[3] = -1
    ora = oracle.apply_policy(pol, idx, tr.tensors, bpo, guard=guard)
    c = make_ctx(P, staging_bytes=max(4096, ora["staging_bytes"]), link_bytes_per_op=bpo, guard_bytes=guard)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    try:
        P.ss_bind(c, arena.data_ptr(), arena_bytes, 0)
        lib = P.ss_apply_policy(c, pol, idx, tr.tensors)
        assert_applied_equal(lib, P, c, ora)
        if ora["staging_bytes"] > 4096:       # too little staging: reported, outputs still complete
            small = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo, guard_bytes=guard)
            try:
                lib = P.ss_apply_policy(small, pol, idx, tr.tensors, allow_nomem=True)
                assert lib["rc"] == P.SS_E_NOMEM and lib["staging_bytes"] == ora["staging_bytes"]
            finally:
                P.ss_destroy(small)
    finally:
        P.ss_destroy(c)
        del arena


def test_apply_policy_keep_late_slow_link(P):
    """a link too slow for the prescribed set: dropped by default, forced around the use with KEEP_LATE"""
    import torch
    tr = W.build_trace(W.config_shape(2))
    pol = W.config_swap_set(tr, 2)
    arena_bytes = place_tensors(tr.tensors)
    idx = pol["ref_op"].astype(np.int64)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    for flags, keep, bin_ in ((0, False, 0), (P.SS_CFG_KEEP_LATE, True, 0), (P.SS_CFG_KEEP_LATE, True, 1 << 20),
                              (0, False, 3 << 20)):
        ora = oracle.apply_policy(pol, idx, tr.tensors, 4 << 20, keep_late=keep, bpo_in=bin_ or None)
        c = make_ctx(P, staging_bytes=max(4096, ora["staging_bytes"]), link_bytes_per_op=4 << 20, flags=flags,
                     prefetch_bytes_per_op=bin_)
        try:
            P.ss_bind(c, arena.data_ptr(), arena_bytes, 0)
            lib = P.ss_apply_policy(c, pol, idx, tr.tensors)
            assert_applied_equal(lib, P, c, ora)
            assert (lib["n_dropped"] == 0) == keep
            n_forced = int(((lib["resolved"]["flags"] & P.SS_F_FORCED) != 0).sum())
            assert n_forced == sum(1 for r in ora["resolved"] if r[3] & oracle.F_FORCED)
            assert (n_forced > 10) == keep
        finally:
            P.ss_destroy(c)


@pytest.mark.parametrize("seed", range(24))
def test_apply_policy_random_tiny_policies_links_and_options(P, seed):
    """a random subset of a tiny random trace as policy (items without a match, a tensor claimed twice),
    a random link share per direction, with and without keeping late items, with and without the
    policy's own points: every output array equal to the oracle's, byte for byte"""
    import torch
    rng = SplitMix64(seed, 31)
    tab, ev = tiny_trace(seed)
    if seed % 2:                  # every other trace with all forward uses before all backward uses
        for i in range(len(tab)):
            tab["last_fwd_use"][i] = min(int(tab["last_fwd_use"][i]), 5)
            tab["first_bwd_use"][i] = max(int(tab["first_bwd_use"][i]), 7)
            tab["free_op"][i] = max(int(tab["free_op"][i]), int(tab["first_bwd_use"][i]))
            tab["alloc_op"][i] = tab["producer_op"][i] = min(int(tab["alloc_op"][i]), int(tab["last_fwd_use"][i]))
    arena_bytes = place_tensors(tab)
    rows = []
    for t in tab:
        if rng.randint(3):
            lf, fb = int(t["last_fwd_use"]), int(t["first_bwd_use"])
            t_free = lf + rng.randint(max(1, fb - lf))
            t_in = min(fb, t_free + 1 + rng.randint(max(1, fb - t_free)))
            rows.append((int(t["producer_op"]), int(t["out_slot"]), int(t["tensor_id"]), 0, lf, t_free, t_in, fb,
                         int(t["nbytes"])))
    if rows and rng.randint(2):
        rows.append(rows[0])
    pol = np.array(rows, dtype=W.POLICY_DT) if rows else np.zeros(0, dtype=W.POLICY_DT)
    idx = np.array([r[0] if rng.randint(6) else -1 for r in rows], dtype=np.int64)
    bpo = [64, 700, 3000, 1 << 40][rng.randint(4)]
    bpo_in = [0, 64, 900][rng.randint(3)]
    keep = bool(rng.randint(2))
    points = bool(rng.randint(2))
    ora = oracle.apply_policy(pol, idx, tab, bpo, keep_late=keep, bpo_in=bpo_in or None, policy_points=points)
    flags = (P.SS_CFG_KEEP_LATE if keep else 0) | (P.SS_CFG_POLICY_POINTS if points else 0)
    c = make_ctx(P, staging_bytes=max(4096, ora["staging_bytes"]), link_bytes_per_op=bpo, prefetch_bytes_per_op=bpo_in,
                 flags=flags)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    try:
        P.ss_bind(c, arena.data_ptr(), arena_bytes, 0)
        lib = P.ss_apply_policy(c, pol, idx, tab)
        assert_applied_equal(lib, P, c, ora)
        assert lib["n_late"] == sum(1 for r in ora["resolved"] if r[3] & oracle.F_LATE
                                    and not r[3] & (oracle.F_UNMATCHED | oracle.F_ORDER))
    finally:
        P.ss_destroy(c)


@pytest.mark.parametrize("seed", range(4))
def test_greedy_policy_tiny(P, seed):
    tab, ev = tiny_trace(seed, n_ops=14, T=8)
    no = oracle.timeline_scan(ev, None, 14, 0, 0)
    c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=INSTANT)
    try:
        for frac in (0.9, 0.75, 0.6):
            budget = int(no["peak"] * frac)
            try:
                rows, ap = oracle.greedy_policy(tab, ev, 14, 0, budget, INSTANT)
            except oracle.Infeasible:
                with pytest.raises(P.SsError) as e:
                    P.ss_greedy_policy(c, tab, ev, 14, 0, budget)
                assert e.value.code == P.SS_E_INFEASIBLE
                continue
            pol, peak = P.ss_greedy_policy(c, tab, ev, 14, 0, budget)
            assert [tuple(int(x) for x in r) for r in pol.tolist()] == rows
            assert peak == oracle.timeline_scan(ev, ap["policy_events"], 14, 0, budget)["peak"] <= budget
    finally:
        P.ss_destroy(c)


def test_greedy_policy_7b_shape_and_apply(P):
    tr = W.build_trace(W.config_shape(3))
    budget, bpo = 48 * 10**9, 256 << 20
    rows, ap0 = oracle.greedy_policy(tr.tensors, tr.events, tr.n_ops, 0, budget, bpo, min_bytes=1 << 20)
    c = make_ctx(P, staging_bytes=4096, link_bytes_per_op=bpo)
    try:
        pol, peak = P.ss_greedy_policy(c, tr.tensors, tr.events, tr.n_ops, 0, budget, min_bytes=1 << 20)
        assert [tuple(int(x) for x in r) for r in pol.tolist()] == rows
        assert peak <= budget
        # arena placement under the policy, then the full schedule
        swapped = {r[2]: (r[5], r[6]) for r in ap0["resolved"]}
        arena_bytes = place_tensors(tr.tensors, swapped=swapped)
        assert arena_bytes <= budget * 1.1
        ora = oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, bpo)
        # 50 GB of staging is not allocated here: the schedule is returned, not loaded
        lib = P.ss_apply_policy(c, pol, pol["ref_op"].astype(np.int32), tr.tensors, allow_nomem=True)
        assert lib["rc"] == P.SS_E_NOMEM
        from helpers import applied_as_arrays
        o = applied_as_arrays(ora)
        for key in ("resolved", "actions", "descs_out", "descs_in", "policy_events"):
            assert np.array_equal(lib[key].view(np.uint8), o[key].view(np.uint8)), key
        assert lib["staging_bytes"] == ora["staging_bytes"] > 40 * 10**9
        assert oracle.schedule_check(ora, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    finally:
        P.ss_destroy(c)
