"""Shared test plumbing: drive the oracle and the HIP library with the same generated inputs."""
import numpy as np

import oracle
import workloads as W


from oracle import events_by_op, ops_tuples                    # noqa: E402,F401
from oracle import record_trace as record_oracle                # noqa: E402,F401
from oracle import execute_schedule as oracle_execute           # noqa: E402,F401


def record_lib(P, ctx, tr):
    P.ss_trace_begin(ctx)
    for i, evs in enumerate(events_by_op(tr)):
        op = P.ss_intern_op(ctx, tr.op_name[i], tr.op_stack[i], tr.op_dtype[i], len(tr.op_outputs[i]),
                            tr.op_phase[i])
        P.ss_trace_record(ctx, op, evs if len(evs) else None)
    return P.ss_trace_view(ctx)


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


class WindowStaging:
    """A staging area of which only the windows ever written are kept, so that oracle.swap_out can
    write a slot at its real offset of a 50 GB staging area without 50 GB of host memory."""

    def __init__(self):
        self.win = {}

    def __setitem__(self, sl, data):
        self.win[(int(sl.start), int(sl.stop))] = np.array(data, dtype=np.uint8, copy=True)

    def __getitem__(self, sl):
        return self.win[(int(sl.start), int(sl.stop))]


class ByteProbe:
    """Byte parity of sampled swapped tensors inside a running iteration, against the oracle.

    For every sampled tensor the bytes of its block are captured on the compute stream right after the
    operator of its last forward use (what swap-out must carry away) and right before the operator of its
    first backward use (what swap-in must have brought back, into dev_off_in).  check() then applies
    oracle.swap_out / oracle.swap_in to the captured source and compares: the staging slot (read through
    ss_host_peek) with the oracle's staging window, the returned block with the oracle's arena block.
    """

    def __init__(self, torch, arena, applied, sample_ids):
        self.torch, self.arena = torch, arena
        res = applied["resolved"]
        self.items = {int(r["tensor_id"]): r for r in res if int(r["tensor_id"]) in sample_ids
                      and not int(r["flags"]) & 3}
        self.d_out = {int(d["tensor_id"]): d for d in applied["descs_out"] if int(d["tensor_id"]) in self.items}
        self.d_in = {int(d["tensor_id"]): d for d in applied["descs_in"] if int(d["tensor_id"]) in self.items}
        self.at_out, self.at_use = {}, {}
        for tid, r in self.items.items():
            self.at_out.setdefault(int(r["t_out"]), []).append(tid)
            self.at_use.setdefault(int(r["t_use"]), []).append(tid)
        self.src, self.back = {}, {}

    def before_op(self, i):
        for tid in self.at_use.get(i, ()):
            d = self.d_in[tid]
            self.back[tid] = self.arena[int(d["dev_off"]):int(d["dev_off"]) + int(d["nbytes"])].clone()

    def after_op(self, i):
        for tid in self.at_out.get(i, ()):
            d = self.d_out[tid]
            self.src[tid] = self.arena[int(d["dev_off"]):int(d["dev_off"]) + int(d["nbytes"])].clone()

    def check(self, P, ctx):
        """after the iteration has drained; returns the number of bytes compared each way"""
        assert set(self.src) == set(self.back) == set(self.items) and self.items
        total = 0
        for tid in sorted(self.items):
            do, di = self.d_out[tid], self.d_in[tid]
            n = int(do["nbytes"])
            src = self.src[tid].cpu().numpy()
            sp = oracle.SparseArena()
            sp.put(int(do["dev_off"]), src)
            st = WindowStaging()
            oracle.swap_out(sp, st, [tuple(int(x) for x in do.tolist())])
            want = st[slice(int(do["host_off"]), int(do["host_off"]) + n)]
            got = P.ss_host_peek(ctx, int(do["host_off"]), n)
            assert np.array_equal(got, want), "staging slot of tensor %d" % tid
            sp2 = oracle.SparseArena()
            oracle.swap_in(sp2, st, [tuple(int(x) for x in di.tolist())])
            assert np.array_equal(self.back[tid].cpu().numpy(), sp2.read(int(di["dev_off"]), n)), \
                "returned block of tensor %d" % tid
            total += n
        return total


def stratified_sample(applied, per_class, seed):
    """tensor ids of swapped tensors: `per_class` of every distinct size, chosen by a seeded shuffle"""
    from workloads.rng import SplitMix64
    by_size = {}
    for d in applied["descs_out"]:
        by_size.setdefault(int(d["nbytes"]), []).append(int(d["tensor_id"]))
    out = set()
    for k, size in enumerate(sorted(by_size)):
        ids = by_size[size]
        perm = SplitMix64(seed, k).permutation(len(ids))
        out.update(ids[j] for j in list(perm)[:per_class])
    return out
