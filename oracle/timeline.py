"""Memory-timeline scan (test oracle).

Sec. 3 (last paragraph): the profiler tracks memory in use at each operator
and logs every swap (place, size), so that the memory curve without swaps can
be rebuilt.  Sec. 4.2: wherever that curve exceeds the limit, a memory
reduction entry (MRE) says by how much.  Sec. 5.2: a swapped-out block is
released right after the operator that is running when the swap-out completes
has been dispatched.

Readings the paper leaves open, fixed here:
 * Memory "at operator t" is the largest amount held at any moment of t: what
   was held on entry plus everything t allocates; what t frees is released
   when t ends.  So inside one operator every allocation precedes every free.
 * A swapped-out tensor's block is released after operator t_free (a free of
   class "policy", the last thing in t_free); its swap-in block is taken
   before operator t_in (an allocation of class "policy", the first thing in
   t_in).  Canonical event order = (operator, class, position in own list)
   with classes: 0 policy alloc, 1 trace alloc, 2 trace free, 3 policy free.
 * `base` stands for everything resident through the whole iteration
   (weights, optimizer state).
"""
import numpy as np


def timeline_scan(events, policy_events, n_ops, base, budget):
    """Walk the events in canonical order with a running total.

    events / policy_events: sequences of (op_idx, tensor_id, delta) (NumPy
    structured arrays or tuples); policy_events may be None.
    Returns dict with
      timeline   int64[E]  running total after each event, canonical order
      per_op     int64[n]  P[t] = largest total during operator t
      mre        int64[n]  max(0, P[t] - budget)
      peak, argpeak_op, n_over, final
    """
    rows = []
    for src, lst in ((0, events), (1, policy_events)):
        if lst is None:
            continue
        for i in range(len(lst)):
            op, tid, delta = int(lst[i][0]), int(lst[i][1]), int(lst[i][2])
            if op >= n_ops:
                raise ValueError("event at operator %d but only %d operators" % (op, n_ops))
            if src == 0:
                cls = 1 if delta >= 0 else 2
            else:
                cls = 0 if delta >= 0 else 3
            rows.append((op, cls, i, delta))
    rows.sort()

    timeline = np.zeros(len(rows), dtype=np.int64)
    per_op = np.zeros(n_ops, dtype=np.int64)
    total = int(base)
    e = 0
    for t in range(n_ops):
        high = total                      # held on entry to operator t
        while e < len(rows) and rows[e][0] == t:
            total += rows[e][3]
            timeline[e] = total
            high = max(high, total)
            e += 1
        per_op[t] = high
    mre = np.maximum(per_op - int(budget), 0)
    if n_ops:
        peak = int(per_op.max())
        argpeak = int(np.argmax(per_op))          # first operator attaining it
    else:
        peak, argpeak = int(base), -1
    return dict(timeline=timeline, per_op=per_op, mre=mre, peak=peak,
                argpeak_op=argpeak, n_over=int((mre > 0).sum()), final=total)
