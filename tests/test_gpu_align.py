"""GPU parity of the sequence aligner (ss_align_sequence, SS_MATCH_ALIGN) against the oracle's
textbook dynamic programme: pairing, LCS length and anchor landings are compared exactly."""
import os

import numpy as np
import pytest

import oracle
from oracle.align import align, align_anchors
import workloads as W
from workloads.rng import SplitMix64
from helpers import record_oracle, ops_tuples

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(__file__)


@pytest.fixture(scope="module")
def P():
    import paper_2509_11076_amd.binding as B
    return B


@pytest.fixture(scope="module")
def ctx(P):
    cfg = P.ss_config_default()
    cfg.staging_bytes = 4096
    c = P.ss_create(cfg)
    yield c
    P.ss_destroy(c)


def ops_arr(keys, n_out=1):
    a = np.zeros(len(keys), dtype=W.OP_DT)
    if len(keys):
        k = np.asarray([ord(x) if isinstance(x, str) else int(x) for x in keys], dtype=np.int64)
        a["op_token"] = 1 + (k % 1000)
        a["stack_hash"] = 7 + k // 1000
        a["sig"] = 0x0101
        a["n_out"] = n_out
    return a


def check(P, ctx, ref, cur, anchors=None):
    lib = P.ss_align_sequence(ctx, ref, cur, anchors)
    ora = align_anchors(ops_tuples(ref), ops_tuples(cur), [] if anchors is None else anchors.tolist())
    assert lib["lcs"] == ora["lcs"] and lib["distance"] == ora["distance"]
    assert np.array_equal(lib["ref_to_cur"], ora["ref_to_cur"])
    assert np.array_equal(lib["new_idx"], ora["new_idx"]) and np.array_equal(lib["level"], ora["level"])
    assert lib["n_unmatched"] == int((ora["new_idx"] < 0).sum())
    return lib


def test_textbook_and_hand_cases(P, ctx):
    for line in open(os.path.join(HERE, "golden", "lcs_textbook.txt")):
        if line.startswith("#") or not line.strip():
            continue
        a, b, want = line.split()
        assert check(P, ctx, ops_arr(a), ops_arr(b))["lcs"] == int(want)
    assert check(P, ctx, ops_arr("ABAB"), ops_arr("AB"))["ref_to_cur"].tolist() == [-1, -1, 0, 1]
    assert check(P, ctx, ops_arr("ACB"), ops_arr("ABC"))["ref_to_cur"].tolist() == [0, -1, 1]
    assert check(P, ctx, ops_arr("XABABABY"), ops_arr("XABABY"))["ref_to_cur"].tolist() == [0, -1, -1, 1, 2, 3, 4, 5]


def test_empty_sequences_anchor_rules_and_limits(P, ctx):
    a = ops_arr("ABCD", n_out=2)
    assert check(P, ctx, a[:0], a)["lcs"] == 0
    assert check(P, ctx, a, a[:0])["ref_to_cur"].tolist() == [-1] * 4
    assert check(P, ctx, a[:0], a[:0])["distance"] == 0
    cur = ops_arr("ACD", n_out=2)
    cur["n_out"][1] = 1
    anchors = np.zeros(7, dtype=W.ANCHOR_DT)
    anchors["ref_op"] = [0, 0, 1, 2, 2, 3, 9]
    anchors["out_slot"] = [0, 1, 0, 0, 1, 1, 0]
    lib = check(P, ctx, a, cur, anchors)
    assert lib["new_idx"].tolist() == [0, 0, -1, 1, -1, 2, -1] and lib["n_keys"] == 3
    # any of the three features makes two operators different; the output count does not
    one = np.zeros(1, dtype=W.OP_DT)
    one[0] = (5, 1, 0x0101, 1)
    for other in ((6, 1, 0x0101, 1), (5, 2, 0x0101, 1), (5, 1, 0x0102, 1)):
        o = one.copy()
        o[0] = other
        assert P.ss_align_sequence(ctx, one, o)["lcs"] == 0
    o[0] = (5, 1, 0x0101, 4)
    assert P.ss_align_sequence(ctx, one, o)["lcs"] == 1
    too_long = np.zeros(65537, dtype=W.OP_DT)
    with pytest.raises(P.SsError) as e:
        P.ss_align_sequence(ctx, too_long, one)
    assert e.value.code == P.SS_E_CAPACITY


@pytest.mark.parametrize("seed", range(12))
def test_random_sequences_across_word_and_block_boundaries(P, ctx, seed):
    """lengths around the 64-bit word (cur) and the 64-row block (ref) boundaries, small alphabets (many
    equally good alignments: the canonical one must come out) and larger ones"""
    rng = SplitMix64(seed, 11)
    sizes = [1, 2, 63, 64, 65, 127, 128, 129, 200, 257, 320]
    n, m = sizes[rng.randint(len(sizes))], sizes[rng.randint(len(sizes))]
    alpha = [1, 2, 3, 8, 40][rng.randint(5)]
    ref = ops_arr([rng.randint(alpha) for _ in range(n)])
    cur = ops_arr([rng.randint(alpha) for _ in range(m)])
    check(P, ctx, ref, cur)
    # a perturbed copy: deletions and insertions of 10 % each
    cur2 = []
    for x in ref["op_token"].tolist():
        if rng.randint(10) == 0:
            cur2.append(500 + rng.randint(3))
        if rng.randint(10) != 0:
            cur2.append(x - 1)
    check(P, ctx, ref, ops_arr(cur2))


def lcs_length_rows(a, b):
    """independent check of the length alone for sizes the oracle's loops are too slow for:
    row-wise table with numpy (running maximum along the row)"""
    a, b = np.asarray(a), np.asarray(b)
    prev = np.zeros(len(b) + 1, dtype=np.int64)
    for x in a:
        t = np.maximum(prev[1:], prev[:-1] + (b == x))
        prev = np.concatenate(([0], np.maximum.accumulate(t)))
    return int(prev[-1])


@pytest.mark.parametrize("n,m,alpha", [(300, 4000, 150), (300, 4200, 90), (200, 9000, 100), (150, 20000, 60), (100, 40000, 200),
                                       (1500, 1500, 2)])
def test_wider_rows_every_word_count_per_lane(P, ctx, n, m, alpha):
    """cur lengths that need 2, 4, 8 and 16 words per lane, with the mask table in global memory as
    well as in LDS; element-by-element against the oracle"""
    rng = SplitMix64(n * 7 + m, 13)
    ref = ops_arr([rng.randint(alpha) for _ in range(n)])
    cur = ops_arr([rng.randint(alpha) for _ in range(m)])
    lib = check(P, ctx, ref, cur)
    assert lib["lcs"] == lcs_length_rows(ref["op_token"], cur["op_token"])


@pytest.mark.parametrize("n,m", [(5000, 5000), (4096, 4097), (65536, 8192), (3000, 65536)])
def test_closed_forms_at_large_sizes(P, ctx, n, m):
    # one repeated key: carries run through every word and lane; the last min(n, m) operators pair
    lib = P.ss_align_sequence(ctx, ops_arr([5] * n), ops_arr([5] * m))
    k = min(n, m)
    assert lib["lcs"] == k and lib["distance"] == n + m - 2 * k
    want = np.full(n, -1, dtype=np.int32)
    want[n - k:] = np.arange(m - k, m)
    assert np.array_equal(lib["ref_to_cur"], want)
    # distinct operators with every 7th dropped and a foreign one inserted after every 5th
    ref_keys = list(range(n))
    cur_keys, where = [], {}
    for x in ref_keys:
        if x % 7 != 3 and len(cur_keys) < m - 1:
            where[x] = len(cur_keys)
            cur_keys.append(x)
            if x % 5 == 0:
                cur_keys.append(100000 + x)
    lib = P.ss_align_sequence(ctx, ops_arr(ref_keys), ops_arr(cur_keys))
    assert lib["lcs"] == len(where)
    assert lib["ref_to_cur"].tolist() == [where.get(x, -1) for x in ref_keys]


def test_random_large_length_and_validity(P, ctx):
    rng = SplitMix64(99, 17)
    n, m = 2500, 7000
    a = [rng.randint(30) for _ in range(n)]
    b = [rng.randint(30) for _ in range(m)]
    lib = P.ss_align_sequence(ctx, ops_arr(a), ops_arr(b))
    assert lib["lcs"] == lcs_length_rows(a, b)
    pairs = [(i, int(j)) for i, j in enumerate(lib["ref_to_cur"]) if j >= 0]
    assert len(pairs) == lib["lcs"] and all(a[i] == b[j] for i, j in pairs)
    assert all(p[0] < q[0] and p[1] < q[1] for p, q in zip(pairs, pairs[1:]))


def test_varying_7b_sequences_and_match_flag(P, ctx):
    """configuration 4's sequences at full size: anchors through ss_align_sequence and through
    ss_match_sequence with SS_MATCH_ALIGN, against the oracle; the similarity verdict is unchanged"""
    shape = W.config_shape(4)
    pert = dict(p_drop=0.1, p_insert=0.1, moe_max=8, seq_jitter=0.15)
    rec = oracle.TraceRecorder()
    tr0 = W.build_trace(shape, iteration=0)
    ref, _ = record_oracle(rec, tr0)
    tab = tr0.tensors
    keep = (tab["first_bwd_use"] != W.NONE_OP) & (tab["last_fwd_use"] != W.NONE_OP)
    anchors = np.zeros(int(keep.sum()), dtype=W.ANCHOR_DT)
    anchors["ref_op"] = tab["producer_op"][keep]; anchors["out_slot"] = tab["out_slot"][keep]
    for it in (1, 2):
        tr1 = W.build_trace(shape, iteration=it, perturb=pert)
        cur, _ = record_oracle(rec, tr1)
        lib = check(P, ctx, ref, cur, anchors)
        assert len(ref) > 1000 and lib["lcs"] > 900 and 0 < lib["n_unmatched"] < len(anchors) // 3
        plain = P.ss_match_sequence(ctx, ref, cur, anchors)
        viaflag = P.ss_match_sequence(ctx, ref, cur, anchors, flags=P.SS_MATCH_ALIGN)
        assert np.array_equal(viaflag["new_idx"], lib["new_idx"]) and np.array_equal(viaflag["level"], lib["level"])
        assert viaflag["n_unmatched"] == lib["n_unmatched"]
        assert (viaflag["similar"], viaflag["dot"], viaflag["na"], viaflag["nb"]) == \
            (plain["similar"], plain["dot"], plain["na"], plain["nb"])
        # against the generator's ground truth the alignment lands right far more often
        truth = {b: j for j, b in enumerate(tr1.op_base) if b is not None}
        t = np.array([truth.get(tr0.op_base[i], -1) for i in anchors["ref_op"].tolist()])
        assert (lib["new_idx"] == t).sum() > 2 * (plain["new_idx"] == t).sum()
