"""GPU: ss_timeline_scan_static (the timeline scan for callers that cannot allocate: scratch in a
static device array, inputs and outputs in the caller's device memory) against ss_timeline_scan
and the oracle, through the C ABI.  Exact equality: everything is integers."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2509_11076_amd.binding as B
    return B


def static_scan(P, torch, ctx, ev, pe, n_ops, base, budget, want_timeline=True, stream=None):
    """device copies in, one enqueue, synchronise, device results out -> dict like binding.ss_timeline_scan"""
    def dev(a):
        if a is None or len(a) == 0:
            return None
        return torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).copy()).cuda()
    d_ev, d_pe = dev(ev), dev(pe)
    n_ev = 0 if ev is None else len(ev)
    n_pe = 0 if pe is None else len(pe)
    # outputs start from a pattern, so that anything the kernel does not write shows
    d_tl = torch.full((max(1, n_ev + n_pe),), -77, dtype=torch.int64, device="cuda") if want_timeline else None
    d_per = torch.full((max(1, n_ops),), -77, dtype=torch.int64, device="cuda")
    d_mre = torch.full((max(1, n_ops),), -77, dtype=torch.int64, device="cuda")
    d_res = torch.full((ctypes.sizeof(P.ss_scan_result_t),), 0xEE, dtype=torch.uint8, device="cuda")
    s = stream if stream is not None else torch.cuda.current_stream()
    s.wait_stream(torch.cuda.current_stream())          # the inputs were produced on the current stream
    P.ss_timeline_scan_static(ctx, s.cuda_stream, d_ev.data_ptr() if d_ev is not None else 0, n_ev,
                              d_pe.data_ptr() if d_pe is not None else 0, n_pe, n_ops, base, budget,
                              d_tl.data_ptr() if d_tl is not None else 0, d_per.data_ptr(), d_mre.data_ptr(),
                              d_res.data_ptr())
    s.synchronize()
    r = P.ss_scan_result_t.from_buffer_copy(d_res.cpu().numpy().tobytes())
    return dict(timeline=None if d_tl is None else d_tl.cpu().numpy()[:n_ev + n_pe], per_op=d_per.cpu().numpy()[:n_ops],
                mre=d_mre.cpu().numpy()[:n_ops], peak=r.peak, argpeak_op=r.argpeak_op, n_over=r.n_over,
                final=r.final_total, sorted=r.sorted, flags=r.reserved)


def assert_same(a, b, timeline=True):
    for k in ("peak", "argpeak_op", "n_over", "final", "sorted"):
        assert a[k] == b[k], k
    assert np.array_equal(a["per_op"], b["per_op"]) and np.array_equal(a["mre"], b["mre"])
    if timeline:
        assert np.array_equal(a["timeline"], b["timeline"])


def test_static_scan_equals_the_allocating_scan_twice_in_a_row_second_smaller(P):
    import torch
    torch.cuda.set_device(0)
    cfg = P.ss_config_default()
    cfg.staging_bytes = 4096
    ctx = P.ss_create(cfg)
    try:
        # first call: the 100,000-event stress trace with the 40,000 events of its whole swap set
        tr, pol, _ = W.build_small_tensor_stress()
        ap = oracle.apply_policy(pol, pol["ref_op"].astype(np.int64), tr.tensors, 256 << 20)
        pe = np.array(ap["policy_events"], dtype=W.EVENT_DT)
        budget = 6 * 10**9
        want = P.ss_timeline_scan(ctx, tr.events, pe, tr.n_ops, 3, budget, want_timeline=True)
        got = static_scan(P, torch, ctx, tr.events, pe, tr.n_ops, 3, budget)
        assert got["flags"] == 0
        assert_same(got, want)
        ora = oracle.timeline_scan(tr.events, pe, tr.n_ops, 3, budget)
        assert got["peak"] == ora["peak"] and np.array_equal(got["timeline"], ora["timeline"])
        # second call, smaller, right after it: the shared scratch still holds the first call's contents
        tr2 = W.build_trace(W.config_shape(2))
        want2 = P.ss_timeline_scan(ctx, tr2.events, None, tr2.n_ops, 7 << 30, 4 << 30, want_timeline=True)
        got2 = static_scan(P, torch, ctx, tr2.events, None, tr2.n_ops, 7 << 30, 4 << 30)
        assert got2["flags"] == 0
        assert_same(got2, want2)
        ora2 = oracle.timeline_scan(tr2.events, None, tr2.n_ops, 7 << 30, 4 << 30)
        assert got2["peak"] == ora2["peak"] and np.array_equal(got2["per_op"], ora2["per_op"])
        assert np.array_equal(got2["timeline"], ora2["timeline"])
        # a third, tiny one on a stream of the caller's own, without a timeline
        tr1 = W.build_trace(W.config_shape(1))
        side = torch.cuda.Stream()
        want1 = P.ss_timeline_scan(ctx, tr1.events, None, tr1.n_ops, 0, 1 << 20)
        got1 = static_scan(P, torch, ctx, tr1.events, None, tr1.n_ops, 0, 1 << 20, want_timeline=False, stream=side)
        assert_same(got1, want1, timeline=False)
    finally:
        P.ss_destroy(ctx)


def test_static_scan_limits_and_kernel_side_errors(P):
    import torch
    torch.cuda.set_device(0)
    cfg = P.ss_config_default()
    cfg.staging_bytes = 4096
    ctx = P.ss_create(cfg)
    try:
        buf = torch.zeros(64, dtype=torch.int64, device="cuda")
        # beyond the stated maximum: refused with a clear code, nothing enqueued
        for n_ev, n_pe, n_ops in ((262145, 0, 10), (200000, 62145, 10), (16, 0, 65537)):
            with pytest.raises(P.SsError) as e:
                P.ss_timeline_scan_static(ctx, 0, buf.data_ptr(), n_ev, buf.data_ptr(), n_pe, n_ops, 0, 0, 0, 0, 0,
                                          buf.data_ptr())
            assert e.value.code == P.SS_E_CAPACITY
        with pytest.raises(P.SsError) as e:                  # the result block is required
            P.ss_timeline_scan_static(ctx, 0, buf.data_ptr(), 1, 0, 0, 1, 0, 0, 0, 0, 0, 0)
        assert e.value.code == P.SS_E_INVAL
        # exactly at the maximum number of operators; empty lists
        got = static_scan(P, torch, ctx, None, None, 65536, 5, 4, want_timeline=False)
        assert got["peak"] == 5 and got["n_over"] == 65536 and got["argpeak_op"] == 0 and got["flags"] == 0
        assert (got["per_op"] == 5).all() and (got["mre"] == 1).all()
        got = static_scan(P, torch, ctx, None, None, 0, 9, 0)
        assert got["peak"] == 9 and got["argpeak_op"] == -1 and got["final"] == 9
        # an event beyond the last operator: flag bit 0 in the result block
        ev = np.zeros(3, dtype=W.EVENT_DT)
        ev["op_idx"] = [0, 1, 7]; ev["delta"] = [4, 4, -8]
        got = static_scan(P, torch, ctx, ev, None, 5, 0, 0)
        assert got["flags"] & 1
        # lists out of operator order: per-operator results valid, sorted = 0, flag bit 1, no timeline written
        ev["op_idx"] = [3, 1, 2]
        got = static_scan(P, torch, ctx, ev, None, 5, 0, 0)
        want = P.ss_timeline_scan(ctx, ev, None, 5, 0, 0)
        assert got["flags"] == 2 and got["sorted"] == 0
        assert_same(got, want, timeline=False)
        assert (got["timeline"] == -77).all()
    finally:
        P.ss_destroy(ctx)
