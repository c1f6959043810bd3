"""Policy application, link timing, greedy policy, schedule checker (test oracle).

Sec. 5 (first paragraph): in the next iteration the executor issues every swap
of the policy at the operator the policy fixed for it.  A policy item names a
tensor (by features of its producing operator, Sec. 5.1) and three points:
where its swap-out is issued (right after its last forward use, Sec. 4.3.2),
where its block is released (after dispatching the operator that is running
when the swap-out completes, Sec. 5.2), and where its swap-in is pre-triggered
so that it completes before the first backward use (Sec. 4.3.1).

The paper's simulator decides those points per logical layer with a remaining-
time budget; that generator is outside this build's hot path.  The stand-in
used here keeps Eq. 3 (T_swap = S / B) and Eq. 1 (every operator is given the
same share of the iteration time) but works at operator granularity with one
FIFO link per direction.  Time is measured in link bytes: operator t occupies
[t * bpo, (t + 1) * bpo) where bpo = B * T_iter / N_iter bytes.

  swap-out queue, items ordered by (t_out, policy index):
      ready = (t_out + 1) * bpo; start = max(ready, link_free);
      end = start + nbytes; link_free = end; t_free = (end - 1) // bpo
  swap-in queue, as late as possible, items ordered by (t_use, policy index)
  descending:
      end = min(t_use * bpo, start of the item placed before); start = end - nbytes
      floor_ = max(t_free + 1, t_peak) * bpo with t_peak = 1 + the largest t_out of the set
      (no swap-in before the last swap-out is issued); if start < floor_: start = floor_, item is LATE
      t_in = start // bpo; finally, walking (t_use, policy index) upwards, t_in = max(t_in, t_in of
      the item before): the swap-in stream is first-in first-out, so an item needed later is never
      issued ahead of one needed earlier
  (the swap-in queue may be given its own bytes-per-operator, bpo_in, in place of bpo:
  a smaller value pre-triggers the swap-ins with more margin)
  An item is valid iff t_out <= t_free < t_in <= t_use.  An item whose swap-out
  cannot complete before its first backward use (t_free >= t_use) saves no
  memory; by default it is dropped (flag ORDER) and keeps no link time in the
  swap-in queue.  With keep_late (a prescribed swap set that must be executed
  whatever it costs; Sec. 4.3.1 accepts latency rather than giving up) it is
  kept instead with t_free = t_use - 1, flags FORCED and LATE: released and
  re-fetched around its use, the compute stream waiting for the round trip.

The paper prints no worked example of its simulator to compare with; pinned by
hand-worked cases, the schedule checker (also on random policies), the live-set
definition of the memory the schedule leaves, and brute force over subsets.
"""
import numpy as np

NONE_OP = 0xFFFFFFFF
K_IN, K_WAIT_IN, K_OUT, K_FREE = 0, 1, 2, 3           # order inside one operator
F_UNMATCHED, F_ORDER, F_LATE, F_RESIZED, F_FORCED = 1, 2, 4, 8, 16


class Infeasible(Exception):
    """No candidate left although memory still exceeds the budget (Algo. 2, the error branch)."""


def _align_up(x, a):
    return (x + a - 1) // a * a


def link_timing(t_out, t_use, nbytes, bpo, keep_late=False, bpo_in=None):
    """Per item: (t_free, t_in, late, valid[, forced]).  Inputs are equal-length integer lists.
    With keep_late a fifth list, forced, is returned as well."""
    k = len(t_out)
    bpo = int(bpo)
    t_free = [0] * k
    t_in = [0] * k
    late = [False] * k
    valid = [True] * k
    forced = [False] * k
    link_free = 0
    for i in sorted(range(k), key=lambda i: (t_out[i], i)):
        ready = (t_out[i] + 1) * bpo
        start = max(ready, link_free)
        end = start + nbytes[i]
        link_free = end
        t_free[i] = (end - 1) // bpo
        if not (t_free[i] < t_use[i]):
            if keep_late:
                t_free[i] = t_use[i] - 1
                forced[i] = True
            else:
                valid[i] = False
    # the swap-in queue may assume another link share per operator (bpo_in): a smaller value
    # stacks the swap-ins earlier, i.e. pre-triggers them with more margin (Sec. 4.3.1)
    bpo = int(bpo_in) if bpo_in else bpo
    # no swap-in is issued before the last swap-out has been issued: before that point memory is
    # still climbing to its peak, and a swap-in there would only fight the swap-outs for the link
    # (Sec. 4.3.1: the search for a swap-in slot does not go back beyond the peak-memory period)
    outs = [t_out[i] for i in range(k) if valid[i]]
    t_peak = max(outs) + 1 if outs else 0
    next_start = None
    for i in sorted(range(k), key=lambda i: (t_use[i], i), reverse=True):
        if not valid[i]:
            continue
        end = t_use[i] * bpo
        if next_start is not None and next_start < end:
            end = next_start
        start = end - nbytes[i]
        floor_ = max(t_free[i] + 1, t_peak) * bpo
        if start < floor_:
            start = floor_
            late[i] = True
        t_in[i] = start // bpo
        next_start = start
    # the swap-in stream is first-in first-out: an item needed later is never issued before one
    # needed earlier (the release-point floor can otherwise put it ahead in the queue)
    run = 0
    for i in sorted(range(k), key=lambda i: (t_use[i], i)):
        if valid[i]:
            t_in[i] = max(t_in[i], run)
            run = t_in[i]
    if keep_late:
        return t_free, t_in, late, valid, forced
    return t_free, t_in, late, valid


def apply_policy(policy, new_idx, tensors, bpo, align=256, guard=0, keep_late=False, bpo_in=None,
                 policy_points=False):
    """Turn a policy plus this iteration's tensor table into the action schedule.

    policy rows: ref_op, out_slot, tensor_id, flags, t_out, t_free, t_in, t_use, nbytes
    new_idx[a]:  operator index in the current iteration producing item a's tensor, or -1
    tensors:     rows with tensor_id, producer_op, out_slot, last_fwd_use, first_bwd_use,
                 dev_off, dev_off_in, nbytes
    Returns dict(resolved, actions, descs_out, descs_in, out_batch_start, in_batch_start,
                 in_dep, policy_events, staging_bytes, n_dropped)
    """
    k = len(policy)
    by_producer = {}
    for row, t in enumerate(tensors):
        by_producer[(int(t["producer_op"]), int(t["out_slot"]))] = row
    cur = [None] * k
    flags = [0] * k
    for a in range(k):
        j = int(new_idx[a])
        row = by_producer.get((j, int(policy[a]["out_slot"]))) if j >= 0 else None
        if row is None:
            flags[a] |= F_UNMATCHED
            continue
        t = tensors[row]
        lf, fb = int(t["last_fwd_use"]), int(t["first_bwd_use"])
        if lf == NONE_OP or fb == NONE_OP or not lf < fb:
            flags[a] |= F_ORDER
            continue
        cur[a] = row
    # one tensor may be claimed once only: the lower policy index keeps it
    seen = set()
    for a in range(k):
        if cur[a] is not None:
            if cur[a] in seen:
                cur[a] = None
                flags[a] |= F_UNMATCHED
            else:
                seen.add(cur[a])
    live = [a for a in range(k) if cur[a] is not None]
    t_out = [int(tensors[cur[a]]["last_fwd_use"]) for a in live]
    t_use = [int(tensors[cur[a]]["first_bwd_use"]) for a in live]
    nb = [int(tensors[cur[a]]["nbytes"]) for a in live]
    if policy_points:
        # the generator already fixed release and pre-trigger points (Sec. 4.3, 4.4): keep them, moved
        # along with the tensor's own last forward use / first backward use in this iteration
        t_free, t_in, late, valid, forced = [], [], [], [], []
        for pos, a in enumerate(live):
            p = policy[a]
            tf = int(p["t_free"]) + t_out[pos] - int(p["t_out"])
            ti = int(p["t_in"]) + t_use[pos] - int(p["t_use"])
            ok = t_out[pos] <= tf < ti <= t_use[pos]
            fz = False
            if not ok and keep_late:
                tf = min(max(tf, t_out[pos]), t_use[pos] - 1)
                ti = min(max(ti, tf + 1), t_use[pos])
                ok, fz = True, True
            t_free.append(tf); t_in.append(ti); valid.append(ok); forced.append(fz)
            late.append(bool(int(p["flags"]) & F_LATE) or fz)
        run = 0                                  # first-in first-out order of need, as in link_timing
        for pos in sorted(range(len(live)), key=lambda q: (t_use[q], live[q])):
            if valid[pos]:
                t_in[pos] = max(t_in[pos], run)
                run = t_in[pos]
    elif keep_late:
        t_free, t_in, late, valid, forced = link_timing(t_out, t_use, nb, bpo, keep_late=True, bpo_in=bpo_in)
    else:
        t_free, t_in, late, valid = link_timing(t_out, t_use, nb, bpo, bpo_in=bpo_in)
        forced = [False] * len(live)

    resolved = []
    kept = []        # (a, row, t_out, t_free, t_in, t_use, nbytes)
    info = {}
    for pos, a in enumerate(live):
        ok = valid[pos] and t_out[pos] <= t_free[pos] < t_in[pos] <= t_use[pos]
        if not ok:
            flags[a] |= F_ORDER
            continue
        if late[pos]:
            flags[a] |= F_LATE
        if forced[pos]:
            flags[a] |= F_FORCED
        if nb[pos] != int(policy[a]["nbytes"]):
            flags[a] |= F_RESIZED
        info[a] = (cur[a], t_out[pos], t_free[pos], t_in[pos], t_use[pos], nb[pos])
        kept.append(a)
    for a in range(k):
        p = policy[a]
        if a in info:
            row, to, tf, ti, tu, n = info[a]
            resolved.append((int(p["ref_op"]), int(p["out_slot"]), int(tensors[row]["tensor_id"]),
                             flags[a], to, tf, ti, tu, n))
        else:
            resolved.append((int(p["ref_op"]), int(p["out_slot"]), int(p["tensor_id"]),
                             flags[a], 0, 0, 0, 0, int(p["nbytes"])))

    out_order = sorted(kept, key=lambda a: (info[a][1], a))            # by (t_out, index)
    in_order = sorted(kept, key=lambda a: (info[a][4], a))             # by (t_use, index)
    out_rank = {a: r for r, a in enumerate(out_order)}
    in_rank = {a: r for r, a in enumerate(in_order)}

    # staging slots in swap-out order
    host_off = {}
    off = guard
    for a in out_order:
        host_off[a] = off
        off += _align_up(info[a][5], align) + guard
    staging_bytes = off if kept else 0

    # batches: all swap-outs issued after the same operator; all swap-ins issued before the same operator
    descs_out, out_batch_start, out_batch_of = [], [0], {}
    prev = None
    for a in out_order:
        row, to = info[a][0], info[a][1]
        if prev is not None and to != prev:
            out_batch_start.append(len(descs_out))
        prev = to
        out_batch_of[a] = len(out_batch_start) - 1
        descs_out.append((int(tensors[row]["dev_off"]), host_off[a], info[a][5],
                          int(tensors[row]["tensor_id"]), flags[a]))
    if kept:
        out_batch_start.append(len(descs_out))
    in_issue = sorted(kept, key=lambda a: (info[a][3], in_rank[a]))    # by (t_in, swap-in order)
    descs_in, in_batch_start, in_batch_of, in_dep = [], [0], {}, []
    prev = None
    for a in in_issue:
        row, ti = info[a][0], (info[a][3], info[a][4])       # a batch: same issue point and same first use
        if prev is not None and ti != prev:
            in_batch_start.append(len(descs_in))
        if prev is None or ti != prev:
            in_dep.append(0)
        prev = ti
        b = len(in_batch_start) - 1
        in_batch_of[a] = b
        in_dep[b] = max(in_dep[b], out_batch_of[a])
        descs_in.append((int(tensors[row]["dev_off_in"]), host_off[a], info[a][5],
                         int(tensors[row]["tensor_id"]), flags[a]))
    if kept:
        in_batch_start.append(len(descs_in))

    actions = []
    for a in kept:
        row, to, tf, ti, tu, n = info[a]
        tid = int(tensors[row]["tensor_id"])
        actions.append(((ti, K_IN, in_rank[a]), (ti, K_IN, tid, in_batch_of[a])))
        actions.append(((tu, K_WAIT_IN, in_rank[a]), (tu, K_WAIT_IN, tid, in_batch_of[a])))
        actions.append(((to, K_OUT, out_rank[a]), (to, K_OUT, tid, out_batch_of[a])))
        actions.append(((tf, K_FREE, out_rank[a]), (tf, K_FREE, tid, out_batch_of[a])))
    actions.sort(key=lambda x: x[0])
    actions = [x[1] for x in actions]

    pe = []
    for a in kept:
        row, to, tf, ti, tu, n = info[a]
        tid = int(tensors[row]["tensor_id"])
        pe.append(((tf, 1, out_rank[a]), (tf, tid, -n)))
        pe.append(((ti, 0, out_rank[a]), (ti, tid, n)))
    pe.sort(key=lambda x: x[0])
    pe = [x[1] for x in pe]

    return dict(resolved=resolved, actions=actions, descs_out=descs_out, descs_in=descs_in,
                out_batch_start=out_batch_start if kept else [0],
                in_batch_start=in_batch_start if kept else [0],
                in_dep=in_dep, policy_events=pe, staging_bytes=staging_bytes,
                n_dropped=k - len(kept))


def greedy_policy(tensors, events, n_ops, base, budget, bpo, min_bytes=0, initial=None,
                  align=256, guard=0, keep_late=False, bpo_in=None):
    """Longest-idle-first swap set that brings the timeline peak within the budget.

    Stand-in for Algo. 2 (Sec. 4.4): the memory reduction list is the set of
    operators whose memory exceeds the budget; candidates are tensors kept from
    forward to backward whose idle span covers at least one such operator and
    which are not "too small" (Sec. 4.2); they are taken longest idle span
    first (then larger first, then lower id) one at a time, the whole set is
    re-timed and the timeline re-scanned, until the peak fits.  No candidate
    left while still over budget raises Infeasible.

    initial: policy rows already in force (e.g. a re-anchored policy that no
    longer suffices); candidates are added on top of them.
    Returns (policy_rows, applied) with policy_rows as tuples
    (ref_op, out_slot, tensor_id, 0, 0, 0, 0, 0, nbytes) and applied the
    apply_policy() result for them.
    """
    from .timeline import timeline_scan

    def identity_idx(rows):
        return [r[0] for r in rows]

    def as_struct(rows):
        a = np.zeros(len(rows), dtype=[("ref_op", "<u4"), ("out_slot", "<u4"), ("tensor_id", "<u4"),
                                       ("flags", "<u4"), ("t_out", "<u4"), ("t_free", "<u4"),
                                       ("t_in", "<u4"), ("t_use", "<u4"), ("nbytes", "<u8")])
        for i, r in enumerate(rows):
            a[i] = r
        return a

    rows = [tuple(int(x) for x in r) for r in (initial if initial is not None else [])]
    applied = apply_policy(as_struct(rows), identity_idx(rows), tensors, bpo, align, guard, keep_late, bpo_in)
    scan = timeline_scan(events, applied["policy_events"], n_ops, base, budget)
    if scan["peak"] <= budget:
        return rows, applied
    over = scan["mre"] > 0
    chosen = {r[2] for r in rows}
    cands = []
    for t in tensors:
        lf, fb, n = int(t["last_fwd_use"]), int(t["first_bwd_use"]), int(t["nbytes"])
        if lf == NONE_OP or fb == NONE_OP or not lf + 1 < fb:
            continue
        if n < min_bytes or int(t["tensor_id"]) in chosen:
            continue
        if not over[lf + 1:fb].any():
            continue
        cands.append((-(fb - lf), -n, int(t["tensor_id"]), int(t["producer_op"]), int(t["out_slot"])))
    cands.sort()
    for (_, negn, tid, prod, slot) in cands:
        rows.append((prod, slot, tid, 0, 0, 0, 0, 0, -negn))
        applied = apply_policy(as_struct(rows), identity_idx(rows), tensors, bpo, align, guard, keep_late, bpo_in)
        scan = timeline_scan(events, applied["policy_events"], n_ops, base, budget)
        if scan["peak"] <= budget:
            return rows, applied
    raise Infeasible("peak %d still above budget %d with all %d candidates swapped"
                     % (scan["peak"], budget, len(cands)))


def schedule_check(applied, tensors, op_inputs, op_outputs):
    """Verify an action schedule from the actions alone.  Returns a list of problems (empty = fine).

    Checks: every kept item has exactly one IN, WAIT_IN, OUT, FREE in that
    causal order; no operator reads or writes a tensor while it is away
    (t_free < t < t_in); staging slots are pairwise disjoint; actions are
    sorted; batches cover the descriptors, hold what their actions say, do not
    mix issue points, and swap-in batches depend on the right swap-out batch.
    """
    problems = []
    acts = applied["actions"]
    keys = [(a[0], a[1]) for a in acts]
    if keys != sorted(keys):
        problems.append("actions not sorted by (operator, kind)")
    per = {}
    for (op, kind, tid, batch) in acts:
        per.setdefault(tid, {}).setdefault(kind, []).append(op)
    away = {}
    for tid, d in per.items():
        if any(len(d.get(kd, [])) != 1 for kd in (K_IN, K_WAIT_IN, K_OUT, K_FREE)):
            problems.append("tensor %d: not exactly one action of each kind" % tid)
            continue
        to, tf, ti, tu = d[K_OUT][0], d[K_FREE][0], d[K_IN][0], d[K_WAIT_IN][0]
        if not (to <= tf < ti <= tu):
            problems.append("tensor %d: order violated %r" % (tid, (to, tf, ti, tu)))
        away[tid] = (tf, ti)
    row_of = {int(t["tensor_id"]): i for i, t in enumerate(tensors)}
    for tid, (tf, ti) in away.items():
        t = tensors[row_of[tid]]
        if int(t["last_fwd_use"]) > per[tid][K_OUT][0]:
            problems.append("tensor %d swapped out before its last forward use" % tid)
        if int(t["first_bwd_use"]) < per[tid][K_WAIT_IN][0]:
            problems.append("tensor %d awaited after its first backward use" % tid)
    for op, (ins, outs) in enumerate(zip(op_inputs, op_outputs)):
        for tid in list(ins) + [x for x in outs if x is not None]:
            if tid in away and away[tid][0] < op < away[tid][1]:
                problems.append("operator %d touches tensor %d while it is swapped out" % (op, tid))
    slots = sorted((d[1], d[1] + d[2]) for d in applied["descs_out"])
    for (a0, a1), (b0, b1) in zip(slots, slots[1:]):
        if b0 < a1:
            problems.append("staging slots overlap: [%d,%d) and [%d,%d)" % (a0, a1, b0, b1))
    if sorted(d[1:4] for d in applied["descs_out"]) != sorted(d[1:4] for d in applied["descs_in"]):
        problems.append("swap-in descriptors do not mirror swap-out descriptors")
    for name, starts, n in (("out", applied["out_batch_start"], len(applied["descs_out"])),
                            ("in", applied["in_batch_start"], len(applied["descs_in"]))):
        if starts[0] != 0 or starts[-1] != n or any(b <= a for a, b in zip(starts, starts[1:])):
            if not (n == 0 and starts == [0]):
                problems.append("%s batches do not partition the descriptors" % name)
                return problems
    # batches: the batch an action names holds that tensor's descriptor; a swap-out batch is what leaves
    # after one operator, a swap-in batch what is issued before one operator for one first use; a
    # swap-in batch depends on the last swap-out batch that holds one of its tensors
    def batch_of(descs, starts):
        out = {}
        for b in range(len(starts) - 1):
            for d in descs[starts[b]:starts[b + 1]]:
                out[d[3]] = b
        return out
    ob = batch_of(applied["descs_out"], applied["out_batch_start"])
    ib = batch_of(applied["descs_in"], applied["in_batch_start"])
    for (op, kind, tid, batch) in acts:
        want = ib.get(tid) if kind in (K_IN, K_WAIT_IN) else ob.get(tid)
        if want != batch:
            problems.append("action %r names batch %d, its descriptor is in batch %r" % ((op, kind, tid), batch, want))
    ok_tids = [tid for tid, d in per.items() if all(len(d.get(kd, [])) == 1 for kd in (K_IN, K_WAIT_IN, K_OUT, K_FREE))]
    for name, table_, key in (("out", ob, lambda d: (d[K_OUT][0],)), ("in", ib, lambda d: (d[K_IN][0], d[K_WAIT_IN][0]))):
        seen, last = {}, None
        for tid in ok_tids:
            if tid in table_:
                seen.setdefault(table_[tid], set()).add(key(per[tid]))
        for b in sorted(seen):
            if len(seen[b]) != 1:
                problems.append("%s batch %d mixes issue points %r" % (name, b, sorted(seen[b])))
            elif last is not None and next(iter(seen[b])) == last:
                problems.append("%s batches %d and %d have the same issue point" % (name, b - 1, b))
            last = next(iter(seen[b])) if len(seen[b]) == 1 else None
    if "in_dep" in applied:
        want = {}
        for tid, b in ib.items():
            if tid in ob:
                want[b] = max(want.get(b, 0), ob[tid])
        got = list(applied["in_dep"])
        if got != [want.get(b, 0) for b in range(len(got))] or len(got) != len(applied["in_batch_start"]) - 1:
            problems.append("swap-in batches depend on %r, their tensors leave in %r" % (got, want))
    return problems
