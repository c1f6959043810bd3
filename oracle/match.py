"""Operator-sequence matcher (test oracle).

Part 1 - similarity verdict and stage machine: Sec. 3 and Algo. 1.  The
sequence of an iteration is compared with the previous one; the stage falls
back to WarmUp only if the length changed by 5 % or more or the cosine
similarity is 95 % or less.  m = 2 and n = 5 (Sec. 6, experimental setup).

Readings fixed here (the paper leaves them open):
 * the length difference is taken relative to the previous sequence:
   20 * |len(cur) - len(prev)| < len(prev); two empty sequences are similar;
 * the cosine is positional: token i of one sequence against token i of the
   other, the shorter one padded with token 0 (reserved, contributes nothing);
 * it is evaluated without floating point: with dot = sum a_i b_i,
   na = sum a_i^2, nb = sum b_i^2, "cos > 0.95" is dot > 0 and
   400 dot^2 > 361 na nb (exact integers);
 * when neither transition of Algo. 1 fires, the stage stays what it was;
 * the step counter is not reset when entering Stable (as printed).

Part 2 - re-anchoring policy items in the current sequence: Sec. 5.1 names
the features (operator name, call stack, data type), asks for tolerance to
minor sequence variation and for integer-only comparison, and gives no
algorithm.  This build's definition, keyed-ordinal matching with feature
relaxation:
   level 0 key = (op_token, stack_hash, sig); level 1 = (op_token, sig);
   level 2 = (op_token).
   For an anchor (ref_op = i, out_slot = s), level by level: K = key of
   ref[i]; r = how many operators before i in ref have key K; j = position of
   the r-th (0-based) operator with key K in cur, if there are that many.
   Accept j if s < cur[j].n_out and the data-type code (low byte of sig)
   equals that of ref[i]; otherwise relax to the next level.
   If several anchors land on the same (j, s), only the one with the lowest
   anchor index keeps it.
"""
import numpy as np

WARMUP, GENPOLICY, STABLE = 0, 1, 2


def similarity(cur_tokens, prev_tokens, histogram=False):
    """Returns (similar, dot, na, nb) with exact integers (na for cur, nb for prev).

    histogram=True is the alternative reading of the cosine: the vectors
    compared are the per-token occurrence counts of the two sequences instead
    of the sequences themselves (insensitive to where an operator was
    inserted).  The length test is the same.
    """
    a = [int(x) for x in cur_tokens]
    b = [int(x) for x in prev_tokens]
    la, lb = len(a), len(b)
    if histogram:
        vocab = max(a + b + [0]) + 1
        ha, hb = [0] * vocab, [0] * vocab
        for x in a:
            ha[x] += 1
        for y in b:
            hb[y] += 1
        ha[0] = hb[0] = 0                         # padding token never counts
        a, b = ha, hb
    dot = sum(x * y for x, y in zip(a, b))        # zip stops at the shorter: padding is 0
    na = sum(x * x for x in a)
    nb = sum(y * y for y in b)
    if la == 0 and lb == 0:
        return True, 0, 0, 0
    len_ok = 20 * abs(la - lb) < lb
    cos_ok = dot > 0 and 400 * dot * dot > 361 * na * nb
    return bool(len_ok and cos_ok), dot, na, nb


class StageMachine:
    """Algo. 1, one call per finished iteration."""

    def __init__(self, m=2, n=5):
        self.m, self.n = m, n
        self.stable_step = 0
        self.prev_stage = WARMUP
        self.prev_tokens = None

    def step(self, tokens):
        tokens = [int(x) for x in tokens]
        if self.prev_tokens is None:          # statics are initialised on the first call
            self.prev_tokens = tokens
        similar = similarity(tokens, self.prev_tokens)[0]
        return self.step_verdict(similar, tokens)

    def step_verdict(self, similar, tokens=None):
        """One finished iteration.  Similar iterations are counted; WarmUp hands over to GenPolicy once
        the count exceeds m (and the count starts again), GenPolicy to Stable once it exceeds n (the
        count runs on); Stable stays.  One dissimilar iteration returns any stage to WarmUp, count 0."""
        if not similar:
            self.prev_stage, self.stable_step = WARMUP, 0
        else:
            self.stable_step += 1
            leave_after = {WARMUP: self.m, GENPOLICY: self.n}.get(self.prev_stage)
            if leave_after is not None and self.stable_step > leave_after:
                if self.prev_stage == WARMUP:
                    self.stable_step = 0
                self.prev_stage = {WARMUP: GENPOLICY, GENPOLICY: STABLE}[self.prev_stage]
        if tokens is not None:
            self.prev_tokens = tokens
        return self.prev_stage


def _key(op, level):
    tok, stack, sig = int(op[0]), int(op[1]), int(op[2])
    return (tok, stack, sig) if level == 0 else (tok, sig) if level == 1 else (tok,)


def match_anchors(ref, cur, anchors):
    """ref, cur: sequences of (op_token, stack_hash, sig, n_out); anchors: (ref_op, out_slot).

    Returns (new_idx int32[k], level uint8[k]); new_idx -1 and level 255 for an
    anchor that finds no place (also for ref_op outside ref).
    """
    k = len(anchors)
    new_idx = np.full(k, -1, dtype=np.int32)
    level = np.full(k, 255, dtype=np.uint8)
    for a in range(k):
        i, s = int(anchors[a][0]), int(anchors[a][1])
        if i >= len(ref):
            continue
        want_dtype = int(ref[i][2]) & 0xFF
        for lv in (0, 1, 2):
            K = _key(ref[i], lv)
            r = 0
            for i2 in range(i):
                if _key(ref[i2], lv) == K:
                    r += 1
            seen = 0
            found = -1
            for j in range(len(cur)):
                if _key(cur[j], lv) == K:
                    if seen == r:
                        found = j
                        break
                    seen += 1
            if found >= 0 and s < int(cur[found][3]) and (int(cur[found][2]) & 0xFF) == want_dtype:
                new_idx[a] = found
                level[a] = lv
                break
    landed = [(int(new_idx[a]), int(anchors[a][1])) for a in range(k)]
    for a in range(k):
        if landed[a][0] < 0:
            continue
        for a2 in range(a):
            if landed[a2] == landed[a]:
                new_idx[a] = -1
                level[a] = 255
                break
    return new_idx, level


def match_sequence(ref, cur, anchors, machine=None, histogram=False):
    """The whole per-iteration call: verdict of cur against ref, stage, anchors."""
    sim, dot, na, nb = similarity([o[0] for o in cur], [o[0] for o in ref], histogram)
    stage = machine.step_verdict(sim) if machine is not None else None
    new_idx, level = match_anchors(ref, cur, anchors)
    return dict(similar=sim, dot=dot, na=na, nb=nb, stage=stage, new_idx=new_idx, level=level,
                n_unmatched=int((new_idx < 0).sum()))
