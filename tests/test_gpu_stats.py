"""GPU: the counters of ss_get_stats against values computed from the outputs they summarise
(anchors per matching level, reuse-interval histogram of the loaded schedule, compute-stream stall)."""
import time

import numpy as np
import pytest

import oracle
import workloads as W
from workloads.arena import place_tensors
from helpers import record_oracle, ops_tuples

pytestmark = pytest.mark.gpu
PERT = dict(p_drop=0.1, p_insert=0.1, moe_max=8, seq_jitter=0.15)


@pytest.fixture(scope="module")
def P():
    import paper_2509_11076_amd.binding as B
    return B


def make_ctx(P, **kw):
    cfg = P.ss_config_default()
    for k, v in kw.items():
        setattr(cfg, k, v)
    return P.ss_create(cfg)


def test_match_level_counters_add_up_to_the_levels_returned(P):
    shape = W.ModelShape("naive", 64, 6, 4, 64, 1, 4, experts0=4)
    tr0 = W.build_trace(shape, iteration=0)
    rec = oracle.TraceRecorder()
    ref, _ = record_oracle(rec, tr0)
    tab = tr0.tensors
    keep = (tab["first_bwd_use"] != W.NONE_OP) & (tab["last_fwd_use"] != W.NONE_OP)
    anchors = np.zeros(int(keep.sum()), dtype=W.ANCHOR_DT)
    anchors["ref_op"] = tab["producer_op"][keep]; anchors["out_slot"] = tab["out_slot"][keep]
    ctx = make_ctx(P, staging_bytes=4096)
    try:
        want = [0] * 5
        for it in range(1, 5):
            cur, _ = record_oracle(rec, W.build_trace(shape, iteration=it, perturb=PERT))
            for flags in (0, P.SS_MATCH_ALIGN):
                m = P.ss_match_sequence(ctx, ref, cur, anchors, flags=flags)
                o = oracle.match_sequence(ops_tuples(ref), ops_tuples(cur), anchors.tolist()) if not flags else \
                    oracle.align_anchors(ops_tuples(ref), ops_tuples(cur), anchors.tolist())
                assert np.array_equal(m["level"], o["level"])
                for lv in o["level"].tolist():
                    want[lv if lv <= 3 else 4] += 1
            a = P.ss_align_sequence(ctx, ref, cur, anchors)
            for lv in a["level"].tolist():
                want[lv if lv <= 3 else 4] += 1
        got = P.ss_get_stats(ctx)["match_levels"]
        assert got == want and want[3] > 0 and want[0] > 0 and sum(want) == 4 * 3 * len(anchors)
    finally:
        P.ss_destroy(ctx)


@pytest.mark.parametrize("cfgno,bpo", [(1, 64 * 1024), (2, 13 << 20)])
def test_reuse_interval_histogram_equals_the_schedule(P, cfgno, bpo):
    import torch
    tr = W.build_trace(W.config_shape(cfgno))
    pol = W.config_swap_set(tr, cfgno)
    idx = pol["ref_op"].astype(np.int64)
    ora = oracle.apply_policy(pol, idx, tr.tensors, bpo, keep_late=True)
    swapped = {r[2]: (r[5], r[6]) for r in ora["resolved"] if not r[3] & 3}
    arena_bytes = place_tensors(tr.tensors, swapped=swapped)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
    ctx = make_ctx(P, staging_bytes=int(ora["staging_bytes"]) + 4096, link_bytes_per_op=bpo, flags=P.SS_CFG_KEEP_LATE)
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
        P.ss_apply_policy(ctx, pol, idx.astype(np.int32), tr.tensors)
        # from the oracle's action list: operators between a tensor's OUT and its FREE
        at = {}
        for (op, kind, tid, b) in ora["actions"]:
            at.setdefault(tid, {})[kind] = op
        gaps = [d[oracle.K_FREE] - d[oracle.K_OUT] for d in at.values()]
        hist = [0] * 16
        for g in gaps:
            hist[min(15, int(np.floor(np.log2(g + 1))))] += 1
        st = P.ss_get_stats(ctx)
        assert st["reuse_hist"] == hist and st["reuse_sum"] == sum(gaps) and st["reuse_count"] == len(gaps) > 0
    finally:
        P.ss_destroy(ctx)


def test_compute_stream_stall_is_the_wait_for_the_batch(P):
    import torch
    n = 256 << 20
    arena = torch.zeros(2 * n, dtype=torch.uint8, device="cuda")
    d = np.zeros(1, dtype=W.DESC_DT)
    d[0] = (0, 0, n, 0, 0)
    start = np.array([0, 1], dtype=np.uint32)
    ctx = make_ctx(P, staging_bytes=n, flags=P.SS_CFG_STALL_TIMING | P.SS_CFG_TIMING)
    try:
        P.ss_bind(ctx, arena.data_ptr(), 2 * n, torch.cuda.current_stream().cuda_stream)
        P.ss_load_schedule(ctx, d, start, d, start)
        # released at once: the compute stream waits for the whole transfer (about 5 ms at link rate)
        P.ss_swap_out(ctx, 0)
        P.ss_sync(ctx, P.SS_SYNC_FREE, 0)
        P.ss_swap_in(ctx, 0)
        P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, 0)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        out_ms, in_ms = P.ss_batch_ms(ctx, 0, 0)[0], P.ss_batch_ms(ctx, 1, 0)[0]
        st = P.ss_get_stats(ctx)
        assert 0.5 * out_ms < st["stall_free_ms"] <= out_ms + 1.0
        assert 0.5 * in_ms < st["stall_wait_in_ms"] <= in_ms + 1.0
        # released only after the host has seen each transfer finished: nothing left to wait for
        P.ss_load_schedule(ctx, d, start, d, start)
        P.ss_swap_out(ctx, 0)
        while not P.ss_batch_done(ctx, 0, 0):
            time.sleep(0.001)
        P.ss_sync(ctx, P.SS_SYNC_FREE, 0)
        P.ss_swap_in(ctx, 0)
        while not P.ss_batch_done(ctx, 1, 0):
            time.sleep(0.001)
        P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, 0)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        st2 = P.ss_get_stats(ctx)
        assert st2["stall_free_ms"] - st["stall_free_ms"] < 0.2
        assert st2["stall_wait_in_ms"] - st["stall_wait_in_ms"] < 0.2
    finally:
        P.ss_destroy(ctx)
    # without the flag nothing is measured
    ctx = make_ctx(P, staging_bytes=n)
    try:
        P.ss_bind(ctx, arena.data_ptr(), 2 * n, torch.cuda.current_stream().cuda_stream)
        P.ss_load_schedule(ctx, d, start, d, start)
        P.ss_swap_out(ctx, 0)
        P.ss_sync(ctx, P.SS_SYNC_FREE, 0)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        assert P.ss_get_stats(ctx)["stall_free_ms"] == 0.0
    finally:
        P.ss_destroy(ctx)
