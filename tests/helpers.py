"""Shared test plumbing: drive the oracle and the HIP library with the same generated inputs."""
import numpy as np

import oracle
import workloads as W


def events_by_op(tr):
    ev = tr.events
    bounds = np.searchsorted(ev["op_idx"], np.arange(tr.n_ops + 1))
    return [ev[bounds[i]:bounds[i + 1]] for i in range(tr.n_ops)]


def record_oracle(rec, tr):
    rec.begin()
    for i, evs in enumerate(events_by_op(tr)):
        op = rec.intern(tr.op_name[i], tr.op_stack[i], tr.op_dtype[i], len(tr.op_outputs[i]), tr.op_phase[i])
        rec.record(op, [tuple(e) for e in evs.tolist()])
    return rec.ops_array(), rec.events_array()


def record_lib(P, ctx, tr):
    P.ss_trace_begin(ctx)
    for i, evs in enumerate(events_by_op(tr)):
        op = P.ss_intern_op(ctx, tr.op_name[i], tr.op_stack[i], tr.op_dtype[i], len(tr.op_outputs[i]),
                            tr.op_phase[i])
        P.ss_trace_record(ctx, op, evs if len(evs) else None)
    return P.ss_trace_view(ctx)


def ops_tuples(ops):
    return [tuple(int(x) for x in o) for o in ops.tolist()]


def applied_as_arrays(ap):
    """oracle.apply_policy result -> arrays laid out like the library's outputs"""
    def arr(rows, dt):
        a = np.zeros(len(rows), dtype=dt)
        for i, r in enumerate(rows):
            a[i] = tuple(r)
        return a
    return dict(resolved=arr(ap["resolved"], W.POLICY_DT), actions=arr(ap["actions"], W.ACTION_DT),
                descs_out=arr(ap["descs_out"], W.DESC_DT), descs_in=arr(ap["descs_in"], W.DESC_DT),
                policy_events=arr(ap["policy_events"], W.EVENT_DT),
                out_start=np.asarray(ap["out_batch_start"], np.uint32),
                in_start=np.asarray(ap["in_batch_start"], np.uint32),
                in_dep=np.asarray(ap["in_dep"], np.uint32))


def assert_applied_equal(lib, P, ctx, ora):
    """lib: dict from binding.ss_apply_policy; ora: oracle.apply_policy result"""
    o = applied_as_arrays(ora)
    for key in ("resolved", "actions", "descs_out", "descs_in", "policy_events"):
        assert lib[key].dtype.itemsize == o[key].dtype.itemsize
        assert np.array_equal(lib[key].view(np.uint8), o[key].view(np.uint8)), key
    assert lib["staging_bytes"] == ora["staging_bytes"]
    assert lib["n_dropped"] == ora["n_dropped"]
    if lib["n_kept"]:
        os_, is_, dep = P.ss_schedule_view(ctx)
        assert np.array_equal(os_, o["out_start"]) and np.array_equal(is_, o["in_start"])
        assert np.array_equal(dep, o["in_dep"])


def oracle_execute(arena, staging, ap, poison=None, writes=None):
    """Sequential reading of an action schedule on NumPy byte arrays.

    ap: oracle.apply_policy result.  poison: byte written over a block at its
    FREE action (or None).  writes: optional dict op_idx -> list of
    (dev_off, bytes) the operator itself writes into the arena.
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
        while i < len(acts) and acts[i][0] == op and acts[i][1] in (oracle.K_IN, oracle.K_WAIT_IN):
            _, kind, tid, b = acts[i]
            if kind == oracle.K_IN and b not in done_in:
                oracle.swap_in(arena, staging, ap["descs_in"][is_[b]:is_[b + 1]])
                done_in.add(b)
            i += 1
        for (off, data) in (writes or {}).get(op, ()):
            arena[off:off + len(data)] = data
        while i < len(acts) and acts[i][0] == op:
            _, kind, tid, b = acts[i]
            if kind == oracle.K_OUT and b not in done_out:
                oracle.swap_out(arena, staging, ap["descs_out"][os_[b]:os_[b + 1]])
                done_out.add(b)
            elif kind == oracle.K_FREE and poison is not None:
                d = d_out[tid]
                arena[d[0]:d[0] + d[2]] = poison
            i += 1
    assert i == len(acts)
