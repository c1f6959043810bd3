"""Pins for the oracle's sequence aligner (longest common subsequence + canonical alignment).  CPU only."""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle.align import lcs_table, align, align_anchors
import workloads as W
from workloads.rng import SplitMix64
from helpers import record_oracle, ops_tuples

HERE = os.path.dirname(__file__)


def ops(keys, n_out=1):
    """sequence of single-letter / integer keys -> operator tuples with distinct (token, stack, sig)"""
    return [(1 + (ord(k) if isinstance(k, str) else int(k)), 7, 0x0101, n_out) for k in keys]


def test_textbook_examples():
    for line in open(os.path.join(HERE, "golden", "lcs_textbook.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a, b, want = line.split()
        r2c, lcs = align(ops(a), ops(b))
        assert lcs == int(want) == int(lcs_table(list(a), list(b))[-1][-1])
        assert int((r2c >= 0).sum()) == lcs


def brute_force_lcs(a, b):
    best = 0
    for r in range(len(a), 0, -1):
        for idx in itertools.combinations(range(len(a)), r):
            it = iter(b)
            if all(any(x == a[i] for x in it) for i in idx):     # is a[idx] a subsequence of b
                return r
    return best


@pytest.mark.parametrize("seed", range(40))
def test_length_against_brute_force_and_alignment_is_valid(seed):
    rng = SplitMix64(seed, 5)
    n, m, alpha = rng.randint(9), rng.randint(11), 1 + rng.randint(4)
    a = [rng.randint(alpha) for _ in range(n)]
    b = [rng.randint(alpha) for _ in range(m)]
    r2c, lcs = align(ops(a), ops(b))
    assert lcs == brute_force_lcs(a, b)
    pairs = [(i, int(j)) for i, j in enumerate(r2c) if j >= 0]
    assert len(pairs) == lcs
    assert all(a[i] == b[j] for i, j in pairs)
    assert all(p[0] < q[0] and p[1] < q[1] for p, q in zip(pairs, pairs[1:]))     # monotone, injective
    # symmetric in its arguments, and the insert/delete edit distance follows
    assert align(ops(b), ops(a))[1] == lcs
    assert align_anchors(ops(a), ops(b), [])["distance"] == n + m - 2 * lcs


def test_closed_forms():
    a = list(range(50))
    assert align(ops(a), ops(a))[1] == 50 and align(ops(a), ops(a))[0].tolist() == a
    assert align(ops(a), ops(a[::-1]))[1] == 1                   # distinct elements reversed
    assert align(ops(a), ops([100 + x for x in a]))[1] == 0      # disjoint alphabets
    assert align(ops([]), ops(a))[1] == 0 and align(ops(a), ops([]))[0].tolist() == [-1] * 50
    # deleting k elements of a sequence of distinct elements: every survivor is paired with itself
    drop = {3, 4, 17, 40, 49}
    b = [x for x in a if x not in drop]
    r2c, lcs = align(ops(a), ops(b))
    assert lcs == 45
    assert [int(j) for i, j in enumerate(r2c) if i not in drop] == list(range(45))
    assert all(r2c[i] == -1 for i in drop)
    # inserting foreign elements anywhere: nothing of the reference is lost
    c = []
    for x in a:
        if x % 7 == 0:
            c += [1000 + x, 2000 + x]
        c.append(x)
    r2c, lcs = align(ops(a), ops(c))
    assert lcs == 50 and [c[j] for j in r2c] == a


def test_canonical_alignment_hand_cases():
    # ABAB against AB: read from the end, equal operators are paired first: the last A, B are taken
    assert align(ops("ABAB"), ops("AB"))[0].tolist() == [-1, -1, 0, 1]
    # ACB against ABC: at (3,3) B != C and L[3][2] = L[3][3] = 2: step left; then B pairs with B; at (2,1)
    # C != A and L[2][0] = 0 < L[2][1] = 1: step up; A pairs with A
    assert align(ops("ACB"), ops("ABC"))[0].tolist() == [0, -1, 1]
    # a repeated layer dropped from the middle cannot be told from one dropped at the front
    assert align(ops("XABABABY"), ops("XABABY"))[0].tolist() == [0, -1, -1, 1, 2, 3, 4, 5]


def test_anchor_rules():
    ref = ops("ABCD", n_out=2)
    cur = [ops("A", 2)[0], ops("C", 1)[0], ops("D", 2)[0]]
    res = align_anchors(ref, cur, [(0, 0), (0, 1), (1, 0), (2, 0), (2, 1), (3, 1), (9, 0)])
    # B is gone; C landed on an operator with one output, so slot 1 finds no place; 9 is outside ref
    assert res["new_idx"].tolist() == [0, 0, -1, 1, -1, 2, -1]
    assert res["level"].tolist() == [3, 3, 255, 3, 255, 3, 255]
    assert res["lcs"] == 3 and res["distance"] == 1
    # keys differ in any of the three features
    a = [(5, 1, 0x0101, 1)]
    for other in ((6, 1, 0x0101, 1), (5, 2, 0x0101, 1), (5, 1, 0x0102, 1)):
        assert align(a, [other])[1] == 0
    assert align(a, [(5, 1, 0x0101, 4)])[1] == 1          # the output count is not part of the key


def test_alignment_beats_keyed_ordinals_on_the_varying_sequences():
    """configuration 4's perturbation (operators dropped and inserted with probability 0.1, branch
    counts changing): how many anchors land on the operator that really is their counterpart"""
    shape = W.ModelShape("naive", 64, 8, 4, 64, 1, 4, experts0=4)
    pert = dict(p_drop=0.1, p_insert=0.1, moe_max=8, seq_jitter=0.15)
    rec = oracle.TraceRecorder()
    tr0 = W.build_trace(shape, iteration=0)
    ref, _ = record_oracle(rec, tr0)
    tab = tr0.tensors
    keep = (tab["first_bwd_use"] != W.NONE_OP) & (tab["last_fwd_use"] != W.NONE_OP)
    anchors = list(zip(tab["producer_op"][keep].tolist(), tab["out_slot"][keep].tolist()))
    right = {"ordinal": 0, "aligned": 0}
    for it in (1, 2, 3):
        tr1 = W.build_trace(shape, iteration=it, perturb=pert)
        cur, _ = record_oracle(rec, tr1)
        truth = {b: j for j, b in enumerate(tr1.op_base) if b is not None}
        o = oracle.match_sequence(ops_tuples(ref), ops_tuples(cur), anchors)["new_idx"]
        al = align_anchors(ops_tuples(ref), ops_tuples(cur), anchors)["new_idx"]
        for a, (i, s) in enumerate(anchors):
            t = truth.get(tr0.op_base[i], -1)
            right["ordinal"] += int(o[a]) == t
            right["aligned"] += int(al[a]) == t
    assert right["aligned"] > 1.5 * right["ordinal"]
    assert right["aligned"] > 0.6 * 3 * len(anchors)
