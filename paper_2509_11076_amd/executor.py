"""Walk one iteration's action schedule around the caller's operators.

Sec. 5 (first paragraph) of the SmartSwap paper: each swap operation of the
policy belongs to one operator of the iteration, and the executor issues it when
the iteration gets there.  This module only sequences calls into libss (swap-out, release, swap-in, wait) around
a caller-supplied `run_op(i)` that enqueues operator i on the compute stream.
It holds no arithmetic of the method.
"""
import numpy as np

from . import binding as B


def batch_lists(actions):
    """Per operator index the (kind, tensor_id, batch) triples, split into what runs before
    and after the operator itself.  actions is the ACTION_DT array from ss_apply_policy, sorted by
    (operator, kind) with IN < WAIT_IN < OUT < FREE, so every (operator, before/after) group is one
    contiguous run of it."""
    before, after = {}, {}
    n = len(actions)
    if n == 0:
        return before, after
    ops = actions["op_idx"].astype(np.int64)
    late = actions["kind"] >= B.SS_ACT_OUT                  # OUT and FREE come after the operator
    group = 2 * ops + late
    cuts = np.flatnonzero(np.diff(group)) + 1
    starts = np.concatenate(([0], cuts)).tolist()
    ends = np.concatenate((cuts, [n])).tolist()
    triples = list(zip(actions["kind"].tolist(), actions["tensor_id"].tolist(), actions["batch"].tolist()))
    gl = group.tolist()
    for s, e in zip(starts, ends):
        g = gl[s]
        (after if g & 1 else before).setdefault(g >> 1, []).extend(triples[s:e])
    return before, after


def run_iteration(ctx, n_ops, actions, run_op, before_after=None):
    """Execute one iteration with one library call per action: for each operator, issue IN / WAIT_IN
    actions, run the operator, then issue OUT / FREE actions; drain the swap streams at the end."""
    before, after = before_after if before_after is not None else batch_lists(actions)
    issued_in, issued_out = set(), set()
    for i in range(n_ops):
        for kind, tid, batch in before.get(i, ()):
            if kind == B.SS_ACT_IN:
                if batch not in issued_in:
                    B.ss_swap_in(ctx, batch)
                    issued_in.add(batch)
            else:
                B.ss_sync(ctx, B.SS_SYNC_WAIT_IN, tid)
        if run_op is not None:
            run_op(i)
        for kind, tid, batch in after.get(i, ()):
            if kind == B.SS_ACT_OUT:
                if batch not in issued_out:
                    B.ss_swap_out(ctx, batch)
                    issued_out.add(batch)
            else:
                B.ss_sync(ctx, B.SS_SYNC_FREE, tid)
    B.ss_sync(ctx, B.SS_SYNC_DRAIN, 0)


def dispatch_points(actions):
    """The operators that have actions before them and those that have actions after them (two sets),
    so that the loop below calls into the library only where something is scheduled."""
    if len(actions) == 0:
        return frozenset(), frozenset()
    late = actions["kind"] >= B.SS_ACT_OUT
    return (frozenset(np.unique(actions["op_idx"][~late]).tolist()),
            frozenset(np.unique(actions["op_idx"][late]).tolist()))


def run_iteration_dispatch(ctx, n_ops, run_op, points, end=None):
    """Execute one iteration of the schedule that the last ss_apply_policy loaded, with ss_dispatch:
    one library call per side of an operator that has actions, the actions themselves issued natively.
    `end`: how the iteration ends, SS_SYNC_DRAIN (the host waits for the swap streams; default) or
    SS_SYNC_ITERATION_END (it does not: the next iteration is ordered behind this one on the device)."""
    before, after = points
    for i in range(n_ops):
        if i in before:
            B.ss_dispatch(ctx, i, 0)
        if run_op is not None:
            run_op(i)
        if i in after:
            B.ss_dispatch(ctx, i, 1)
    B.ss_sync(ctx, B.SS_SYNC_DRAIN if end is None else end, 0)
