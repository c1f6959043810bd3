"""Sequence aligner (test oracle): longest common subsequence of two operator sequences and the
canonical alignment read off its table.

Sec. 5.1 asks the matcher to tolerate minor variations of the operator sequence and to compare
integers only; it gives no algorithm.  Keyed-ordinal matching (match_anchors) mislands when an
operator with the anchor's own key is dropped or inserted earlier in the sequence, because every later
ordinal shifts.  Aligning the two sequences as a whole does not: this module is the textbook
dynamic programme for the longest common subsequence (equivalently the edit distance with insertions
and deletions only, n + m - 2 LCS), written out plainly.

Definitions fixed here (this build's: the paper has no aligner; pinned by textbook examples, brute
force over all subsequences and closed forms):
 * two operators are equal when (op_token, stack_hash, sig) are equal;
 * L[i][j] = LCS length of ref[:i] and cur[:j];
   L[i][j] = L[i-1][j-1] + 1 if ref[i-1] == cur[j-1] else max(L[i-1][j], L[i][j-1]);
 * of the many optimal alignments the canonical one is read from (n, m) backwards: equal operators
   are paired (step to (i-1, j-1)); otherwise step left (j-1) if L[i][j-1] == L[i][j], else up (i-1);
 * an anchor (ref_op, out_slot) lands on the operator its ref_op is paired with, provided that
   operator has more than out_slot outputs; otherwise it finds no place (-1).  Level code 3.
"""
import numpy as np

LEVEL_ALIGN = 3


def _keys(ops):
    return [(int(o[0]), int(o[1]), int(o[2])) for o in ops]


def lcs_table(a, b):
    """textbook table, (len(a)+1) x (len(b)+1)"""
    n, m = len(a), len(b)
    L = np.zeros((n + 1, m + 1), dtype=np.int64)
    for i in range(1, n + 1):
        ai = a[i - 1]
        row, prev = L[i], L[i - 1]
        for j in range(1, m + 1):
            if ai == b[j - 1]:
                row[j] = prev[j - 1] + 1
            else:
                row[j] = prev[j] if prev[j] >= row[j - 1] else row[j - 1]
    return L


def align(ref, cur):
    """ref, cur: sequences of (op_token, stack_hash, sig, n_out).  Returns (ref_to_cur int32[n], lcs)."""
    a, b = _keys(ref), _keys(cur)
    L = lcs_table(a, b)
    n, m = len(a), len(b)
    ref_to_cur = np.full(n, -1, dtype=np.int32)
    i, j = n, m
    while i > 0 and j > 0:
        if a[i - 1] == b[j - 1]:
            ref_to_cur[i - 1] = j - 1
            i, j = i - 1, j - 1
        elif L[i][j - 1] == L[i][j]:
            j -= 1
        else:
            i -= 1
    return ref_to_cur, int(L[n][m])


def align_anchors(ref, cur, anchors):
    """Returns dict(new_idx int32[k], level uint8[k], ref_to_cur, lcs, distance)."""
    ref_to_cur, lcs = align(ref, cur)
    k = len(anchors)
    new_idx = np.full(k, -1, dtype=np.int32)
    level = np.full(k, 255, dtype=np.uint8)
    for a in range(k):
        i, s = int(anchors[a][0]), int(anchors[a][1])
        if i < len(ref) and ref_to_cur[i] >= 0 and s < int(cur[int(ref_to_cur[i])][3]):
            new_idx[a] = ref_to_cur[i]
            level[a] = LEVEL_ALIGN
    return dict(new_idx=new_idx, level=level, ref_to_cur=ref_to_cur, lcs=lcs,
                distance=len(ref) + len(cur) - 2 * lcs)
