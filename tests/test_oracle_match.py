"""Pins for the oracle's similarity verdict, stage machine and anchor matcher (CPU only)."""
import os

import numpy as np
import pytest

import oracle
import workloads as W
from workloads.rng import SplitMix64
from test_oracle_trace_timeline import record_trace

GOLD = os.path.join(os.path.dirname(__file__), "golden")
STAGE = {"WarmUp": oracle.WARMUP, "GenPolicy": oracle.GENPOLICY, "Stable": oracle.STABLE}


def golden_stage_cases():
    cases = {}
    for line in open(os.path.join(GOLD, "stage_machine_m2_n5.txt")):
        if line.startswith("#") or not line.strip():
            continue
        c, it, sim, step, stage = line.split()
        cases.setdefault(c, []).append((int(sim), int(step), STAGE[stage]))
    return cases


@pytest.mark.parametrize("case", sorted(golden_stage_cases()))
def test_stage_machine_against_hand_derived_table(case):
    sm = oracle.StageMachine(m=2, n=5)
    for sim, step, stage in golden_stage_cases()[case]:
        assert sm.step_verdict(bool(sim)) == stage
        assert sm.stable_step == step


def test_stage_machine_first_call_compares_sequence_with_itself():
    sm = oracle.StageMachine()
    assert sm.step([5, 6, 7]) == oracle.WARMUP and sm.stable_step == 1
    assert sm.step([9, 9, 9, 9, 9, 9]) == oracle.WARMUP and sm.stable_step == 0   # length doubled


def test_cosine_threshold_is_exact_and_strict():
    # cos = 19/20 exactly: not similar (strict >); one more on the aligned component: similar
    a = [1, 0, 0, 0, 0]
    sim, dot, na, nb = oracle.similarity(a, [19, 5, 3, 2, 1])
    assert (dot, na, nb) == (19, 1, 400) and not sim
    sim, dot, na, nb = oracle.similarity(a, [20, 5, 3, 2, 1])
    assert (dot, na, nb) == (20, 1, 439) and sim        # 400*400 > 361*439
    assert oracle.similarity([3, 1, 4, 1, 5], [3, 1, 4, 1, 5])[0]      # identical: dot^2 == na*nb
    assert not oracle.similarity([1, 2], [0, 0])[0]                   # zero vector


def test_length_test_is_strict_and_relative_to_previous():
    base = [1] * 100
    assert oracle.similarity([1] * 104, base)[0]          # 4 % longer
    assert not oracle.similarity([1] * 105, base)[0]      # 5 %: refused (strict <)
    assert oracle.similarity([1] * 96 + [0] * 0, base)[0]
    assert not oracle.similarity([1] * 95, base)[0]
    assert oracle.similarity([], [])[0] and not oracle.similarity([1], [])[0]


@pytest.mark.parametrize("seed", range(5))
def test_cosine_agrees_with_float64_library_routine_away_from_threshold(seed):
    rng = SplitMix64(seed, 3)
    n = 200
    a = [1 + rng.randint(40) for _ in range(n)]
    b = list(a)
    for _ in range(rng.randint(60)):
        b[rng.randint(n)] = 1 + rng.randint(40)
    sim, dot, na, nb = oracle.similarity(a, b)
    fa, fb = np.array(a, float), np.array(b, float)
    cos = float(fa @ fb / (np.linalg.norm(fa) * np.linalg.norm(fb)))
    assert dot == int(fa @ fb) and na == int(fa @ fa) and nb == int(fb @ fb)
    if abs(cos - 0.95) > 1e-9:
        assert sim == (cos > 0.95)


def test_histogram_reading_ignores_position():
    a = [1, 2, 3, 4, 5, 6, 7, 8] * 10
    b = a[3:] + a[:3]                        # rotation: same multiset of operators
    assert oracle.similarity(a, b, histogram=True)[0]
    sim, dot, na, nb = oracle.similarity([1, 1, 2], [1, 2, 2], histogram=True)
    assert (dot, na, nb) == (2 * 1 + 1 * 2, 5, 5)


def test_cosine_sums_do_not_overflow_for_long_sequences():
    n = 1 << 16
    a = [(1 << 17) + (i % 7) for i in range(n)]
    sim, dot, na, nb = oracle.similarity(a, a)
    assert dot == na == nb and dot > 1 << 50 and sim


# ----------------------------------------------------------------- anchors
def online_counter_match(ref, cur, anchors):
    """Independent formulation: what a dispatch hook would do.  One counter per
    key, bumped at every dispatch; an anchor fires when its key's counter equals
    the anchor's occurrence ordinal in the reference sequence."""
    def keys(op):
        return ((0, op[0], op[1], op[2]), (1, op[0], op[2]), (2, op[0]))
    ordinal = {}
    cnt = {}
    for i, op in enumerate(ref):
        for K in keys(op):
            ordinal[(i, K[0])] = cnt.get(K, 0)
            cnt[K] = cnt.get(K, 0) + 1
    hits = [[None] * 3 for _ in anchors]
    cnt = {}
    for j, op in enumerate(cur):
        for K in keys(op):
            c = cnt.get(K, 0)
            for a, (i, s) in enumerate(anchors):
                if i < len(ref) and keys(ref[i])[K[0]] == K and ordinal[(i, K[0])] == c:
                    hits[a][K[0]] = j
            cnt[K] = c + 1
    out = []
    for a, (i, s) in enumerate(anchors):
        got = -1
        for lv in range(3):
            j = hits[a][lv]
            if j is not None and s < cur[j][3] and (cur[j][2] & 0xFF) == (ref[i][2] & 0xFF):
                got = j
                break
        out.append(got)
    taken = {}
    for a, j in enumerate(out):
        if j >= 0:
            key = (j, anchors[a][1])
            if key in taken:
                out[a] = -1
            else:
                taken[key] = a
    return out


def ops_of(tr, rec=None):
    rec = rec or oracle.TraceRecorder()
    ops, _ = record_trace(rec, tr)
    return [tuple(int(x) for x in o) for o in ops.tolist()], rec


def test_identical_sequence_anchors_stay_put():
    tr = W.build_trace(W.config_shape(1))
    ops, _ = ops_of(tr)
    pol = W.config_swap_set(tr, 1)
    anchors = [(int(p["ref_op"]), int(p["out_slot"])) for p in pol]
    idx, lvl = oracle.match_anchors(ops, ops, anchors)
    assert idx.tolist() == [a[0] for a in anchors] and (lvl == 0).all()


def test_inserted_and_dropped_foreign_operators_do_not_move_anchors():
    """the failure case of index-based identification (Sec. 6.3): extra operators appear"""
    tr = W.build_trace(W.config_shape(1))
    ops, _ = ops_of(tr)
    pol = W.config_swap_set(tr, 1)
    anchors = [(int(p["ref_op"]), int(p["out_slot"])) for p in pol]
    anchor_keys = {ops[i][:3] for (i, _) in anchors}
    rng = SplitMix64(11)
    cur, truth = [], {}
    for i, op in enumerate(ops):
        if rng.bernoulli(0.3):
            cur.append((900 + rng.randint(5), 77, 2, 1))            # validation-like extra operator
        if op[:3] not in anchor_keys and rng.bernoulli(0.3):
            continue                                                # e.g. a skipped optimizer step
        truth[i] = len(cur)
        cur.append(op)
    idx, lvl = oracle.match_anchors(ops, cur, anchors)
    assert idx.tolist() == [truth[i] for (i, _) in anchors] and (lvl == 0).all()
    # positional identification would have failed
    assert any(cur[i][:3] != ops[i][:3] for (i, _) in anchors if i < len(cur))


@pytest.mark.parametrize("it", range(1, 5))
def test_perturbed_sequences_match_is_injective_monotone_and_equals_online_form(it):
    shape = W.ModelShape("naive", 64, 4, 4, 64, 1, 4, experts0=4)
    pert = dict(p_drop=0.1, p_insert=0.1, moe_max=8, seq_jitter=0.15)
    tr0 = W.build_trace(shape, iteration=0)
    tr1 = W.build_trace(shape, iteration=it, perturb=pert)
    ref, rec = ops_of(tr0)
    cur, _ = ops_of(tr1, rec)
    tab = tr0.tensors
    keep = (tab["first_bwd_use"] != W.NONE_OP) & (tab["last_fwd_use"] != W.NONE_OP)
    anchors = [(int(t["producer_op"]), int(t["out_slot"])) for t in tab[keep]]
    idx, lvl = oracle.match_anchors(ref, cur, anchors)
    assert idx.tolist() == online_counter_match(ref, cur, anchors)
    landed = [(j, s) for j, (_, s) in zip(idx.tolist(), anchors) if j >= 0]
    assert len(landed) == len(set(landed))
    # within one key class and level, reference order is preserved
    by_key = {}
    for a, (i, s) in enumerate(anchors):
        if idx[a] >= 0 and lvl[a] == 0:
            by_key.setdefault((ref[i][:3], s), []).append((i, int(idx[a])))
    for pairs in by_key.values():
        pairs.sort()
        assert [j for _, j in pairs] == sorted(j for _, j in pairs)
    # every matched operator carries the anchor's operator name and data type
    for a, (i, s) in enumerate(anchors):
        if idx[a] >= 0:
            assert cur[idx[a]][0] == ref[i][0] and cur[idx[a]][2] & 0xFF == ref[i][2] & 0xFF
            assert s < cur[idx[a]][3]
    assert (idx >= 0).mean() > 0.5


def test_relaxation_levels_and_rejections():
    ref = [(1, 10, 0x101, 1), (1, 10, 0x101, 1), (2, 20, 0x201, 2)]
    # same name, other call stack -> level 1; other sig too -> level 2; other dtype -> no match
    cur = [(1, 11, 0x101, 1), (1, 12, 0x10101, 1), (2, 20, 0x202, 2)]
    idx, lvl = oracle.match_anchors(ref, cur, [(0, 0), (1, 0), (2, 1), (2, 5), (7, 0)])
    # anchor 0: no operator with its call stack, level 1 finds cur[0].
    # anchor 1: ordinal 1 of key (1, 0x101) does not exist in cur, level 2 (name only) finds cur[1],
    #           whose data-type code is still 1.
    # anchor 2: only the name matches and the data type differs; anchor 3: slot 5 of a 2-output
    #           operator; anchor 4: outside the reference.
    assert idx.tolist() == [0, 1, -1, -1, -1]
    assert lvl.tolist() == [1, 2, 255, 255, 255]


def test_injectivity_lower_anchor_index_wins():
    ref = [(1, 1, 1, 1), (1, 2, 1, 1)]
    cur = [(1, 3, 1, 1)]
    # both anchors relax: anchor 0 lands on cur[0] at level 1; anchor 1 has ordinal 1 -> none
    idx, lvl = oracle.match_anchors(ref, cur, [(0, 0), (1, 0), (0, 0)])
    assert idx.tolist() == [0, -1, -1]
