"""Sequencing of the oracle's functions over a whole iteration (test oracle; no arithmetic here).

The functions of this package each restate one step; a parity check, the smoke run and the
CPU-baseline leg of the benchmark need them strung together the way a dispatch loop would:
record every operator of a generated trace, then walk the action schedule of apply_policy in
operator order and move the bytes at each action.  Nothing is computed here that the step
functions do not define.
"""
import numpy as np

from .policy import K_IN, K_WAIT_IN, K_OUT, K_FREE
from .swap import swap_in, swap_out


def events_by_op(tr):
    """the trace generator's event list cut per operator (events are in operator order)"""
    ev = tr.events
    bounds = np.searchsorted(ev["op_idx"], np.arange(tr.n_ops + 1))
    return [ev[bounds[i]:bounds[i + 1]] for i in range(tr.n_ops)]


def record_trace(rec, tr):
    """Sec. 3: every operator of the generated trace `tr` through TraceRecorder `rec`"""
    rec.begin()
    for i, evs in enumerate(events_by_op(tr)):
        op = rec.intern(tr.op_name[i], tr.op_stack[i], tr.op_dtype[i], len(tr.op_outputs[i]), tr.op_phase[i])
        rec.record(op, [tuple(e) for e in evs.tolist()])
    return rec.ops_array(), rec.events_array()


def ops_tuples(ops):
    return [tuple(int(x) for x in o) for o in ops.tolist()]


def execute_schedule(arena, staging, ap, poison=None, writes=None):
    """Sequential reading of an action schedule on byte arrays (Sec. 5: every swap is
    issued at the operator its policy item fixed; inside one operator IN and WAIT_IN come before it,
    OUT and FREE after it).

    ap: apply_policy result.  poison: byte written over a block at its FREE action (or None).
    writes: optional dict op_idx -> list of (dev_off, bytes) the operator itself writes.
    """
    os_, is_ = ap["out_batch_start"], ap["in_batch_start"]
    d_out = {d[3]: d for d in ap["descs_out"]}
    done_out, done_in = set(), set()
    acts = ap["actions"]
    i = 0
    n_ops = (max(a[0] for a in acts) + 1) if acts else 0
    if writes:
        n_ops = max(n_ops, max(writes) + 1)
    for op in range(n_ops):
        while i < len(acts) and acts[i][0] == op and acts[i][1] in (K_IN, K_WAIT_IN):
            _, kind, tid, b = acts[i]
            if kind == K_IN and b not in done_in:
                swap_in(arena, staging, ap["descs_in"][is_[b]:is_[b + 1]])
                done_in.add(b)
            i += 1
        for (off, data) in (writes or {}).get(op, ()):
            arena[off:off + len(data)] = data
        while i < len(acts) and acts[i][0] == op:
            _, kind, tid, b = acts[i]
            if kind == K_OUT and b not in done_out:
                swap_out(arena, staging, ap["descs_out"][os_[b]:os_[b + 1]])
                done_out.add(b)
            elif kind == K_FREE and poison is not None:
                d = d_out[tid]
                arena[d[0]:d[0] + d[2]] = poison
            i += 1
    assert i == len(acts)
