"""GPU parity of the staged swap-out path (SS_PATH_STAGED: copy kernel gathers batches into an HBM ring,
one copy-engine transfer per ring group carries them to the staging area) against the oracle's byte
copies and against the run without swapping."""
import numpy as np
import pytest

import oracle
import workloads as W
from workloads.arena import place_tensors
from helpers import oracle_execute, assert_applied_equal

pytestmark = pytest.mark.gpu
INSTANT = 1 << 40


@pytest.fixture(scope="module")
def P():
    import paper_2509_11076_amd.binding as B
    return B


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


def make_ctx(P, **kw):
    cfg = P.ss_config_default()
    for k, v in kw.items():
        setattr(cfg, k, v)
    return P.ss_create(cfg)


def random_arena(torch, nbytes, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    a = torch.randint(-2**62, 2**62, ((nbytes + 7) // 8,), dtype=torch.int64, device="cuda", generator=g)
    return a.view(torch.uint8)[:nbytes]


@pytest.mark.parametrize("bpo", [64 * 1024, INSTANT])
@pytest.mark.parametrize("slot_kib,slots", [(512, 2), (1024, 3), (4096, 2)])
@pytest.mark.parametrize("staged_in,taper", [(False, 0), (True, 0), (True, 1), (True, 4)])
@pytest.mark.parametrize("bare", [False, True])
def test_toy_config_through_the_ring(P, torch, bpo, slot_kib, slots, staged_in, taper, bare):
    """configuration 1 with ring slots smaller than, about, and larger than a layer's swap set: staging
    image and arena (with poison over released blocks) equal the oracle's, byte for byte; the same with the
    ring transfers issued bare by the library's own thread (SS_CFG_BARE_RING)"""
    from paper_2509_11076_amd.executor import run_iteration
    tr = W.build_trace(W.config_shape(1))
    pol = W.config_swap_set(tr, 1)
    idx = pol["ref_op"].astype(np.int64)
    ap0 = oracle.apply_policy(pol, idx, tr.tensors, bpo)
    swapped = {r[2]: (r[5], r[6]) for r in ap0["resolved"] if not r[3] & 3}
    arena_bytes = place_tensors(tr.tensors, swapped=swapped)
    ora = oracle.apply_policy(pol, idx, tr.tensors, bpo)
    arena = random_arena(torch, arena_bytes, 2509)
    host_arena = arena.cpu().numpy().copy()
    ctx = make_ctx(P, staging_bytes=ora["staging_bytes"], link_bytes_per_op=bpo, copy_path=P.SS_PATH_STAGED,
                   copy_path_in=P.SS_PATH_STAGED if staged_in else P.SS_PATH_AUTO,
                   ring_slot_bytes=slot_kib << 10, ring_bytes=slots * (slot_kib << 10), ring_taper=taper,
                   flags=P.SS_CFG_POISON_FREE | P.SS_CFG_TIMING | (P.SS_CFG_BARE_RING if bare else 0))
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
        for it in range(2):                     # the second iteration re-uses ring slots and event sets
            lib = P.ss_apply_policy(ctx, pol, idx, tr.tensors)
            assert_applied_equal(lib, P, ctx, ora)
            group_of, group_bytes = P.ss_ring_view(ctx)
            assert (group_of >= 0).all() and len(group_bytes) >= 1 and int(group_bytes.max()) <= slot_kib << 10
            assert int(group_bytes.sum()) == sum(d[2] for d in ora["descs_out"])
            P.ss_staging_fill(ctx, 0xA5)
            staging = np.full(ora["staging_bytes"], 0xA5, dtype=np.uint8)
            run_iteration(ctx, tr.n_ops, lib["actions"], None)
            torch.cuda.synchronize()
            oracle_execute(host_arena, staging, ora, poison=0xDB)
            assert np.array_equal(P.ss_host_peek(ctx, 0, ora["staging_bytes"]), staging)
            assert np.array_equal(arena.cpu().numpy(), host_arena)
            for g in range(len(group_bytes)):
                # bare: on the host's clock, where two short transfers may be seen complete in the same look
                assert P.ss_batch_ms(ctx, 2, g)[0] >= 0 if bare else P.ss_batch_ms(ctx, 2, g)[0] > 0
            assert P.ss_batch_ms(ctx, 2)[1] > 0 and P.ss_batch_ms(ctx, 0, 0)[0] > 0
            if bare:                                   # no events on the transfers: nothing to place them among the batches
                with pytest.raises(P.SsError) as ei:
                    P.ss_batch_window(ctx, 2, 0)
                assert ei.value.code == P.SS_E_STATE
            else:
                w = P.ss_batch_window(ctx, 2, 0)
                assert w[1] > w[0] >= 0
            # the same durations, every unit of a direction in one call
            for dr, n_units in ((0, lib["n_out_batches"]), (1, lib["n_in_batches"]), (2, len(group_bytes))):
                all_ms = P.ss_batch_ms_all(ctx, dr)
                assert len(all_ms) == n_units
                assert all_ms.tolist() == [np.float32(P.ss_batch_ms(ctx, dr, u)[0]) for u in range(n_units)]
            in_group_of, in_group_bytes = P.ss_ring_view(ctx, 1)
            if staged_in:
                assert (in_group_of >= 0).all() and int(in_group_bytes.sum()) == int(group_bytes.sum())
                assert int(in_group_bytes.max()) <= slot_kib << 10
                for g in range(len(in_group_bytes)):
                    assert P.ss_batch_ms(ctx, 3, g)[0] >= 0 if bare else P.ss_batch_ms(ctx, 3, g)[0] > 0
                # group shapes: tapered, each swap-in group (of more than one batch) is at most half (a taper of
                # n >= 2: 1/n) of what is still to come including itself, but never asked to be smaller than an
                # eighth of a slot;
                # untapered, a group ends only where the next batch would overflow the slot or leave a gap
                sizes = in_group_bytes.tolist()
                batches_in = np.bincount(in_group_of, minlength=len(sizes)).tolist()
                for g, n in enumerate(sizes):
                    cap = max((slot_kib << 10) // 8, min(sum(sizes[g:]) // max(2, taper), sum(sizes[:g])))
                    if taper != 1 and batches_in[g] > 1:
                        assert n <= cap
                if taper == 1 and sum(sizes) > slot_kib << 10:
                    assert max(sizes) > (slot_kib << 10) // 2
                out_sizes = group_bytes.tolist()
                batches_out = np.bincount(group_of, minlength=len(out_sizes)).tolist()
                for g, n in enumerate(out_sizes):
                    if taper != 1 and batches_out[g] > 1:
                        assert n <= max((slot_kib << 10) // 8, sum(out_sizes[:g]))
            else:
                assert len(in_group_bytes) == 0 and (in_group_of == -1).all()
        st = P.ss_get_stats(ctx)
        assert (st["ring_batches_in"] == 2 * lib["n_in_batches"]) == staged_in
        assert (st["ring_transfers_in"] == 2 * len(in_group_bytes)) and (st["ring_transfers_in"] > 0) == staged_in
        assert st["ring_batches"] == 2 * lib["n_out_batches"] and st["ring_transfers"] >= 2 * len(group_bytes)
        assert st["bytes_out"] == st["bytes_in"] == 2 * sum(d[2] for d in ora["descs_out"])
    finally:
        P.ss_destroy(ctx)


def test_ring_takes_only_gap_free_batches_and_the_rest_leaves_directly(P, torch):
    """a schedule mixing batches the ring can take (sizes multiples of the alignment, consecutive slots)
    with ragged ones and one larger than a slot; batches issued out of order; a release between the gather
    and the transfer; swap-ins that need a group before it is complete"""
    KiB = 1 << 10
    sizes = [256 * KiB, 512 * KiB, 256 * KiB,          # batches 0, 1, 2: one group (slot 1 MiB)
             300 * KiB + 5,                            # batch 3: ragged -> direct
             256 * KiB, 256 * KiB,                     # batch 4 (two tensors): a group of its own with batch 5?
             768 * KiB,                                # batch 5: fits the same slot together with batch 4? 512 + 768 > 1024 -> new group
             2048 * KiB,                               # batch 6: larger than a slot -> direct
             128 * KiB, 128 * KiB]                     # batches 7, 8: one group
    starts = [0, 1, 2, 3, 4, 6, 7, 8, 9, 10]
    n = len(sizes)
    d = np.zeros(n, dtype=W.DESC_DT)
    off = h = 0
    for i, sz in enumerate(sizes):
        d[i] = (off, h, sz, i, 0)
        off += (sz + 4095) // 4096 * 4096 + 4096
        h += (sz + 255) // 256 * 256
    arena_bytes = off
    arena = random_arena(torch, arena_bytes, 9)
    host = arena.cpu().numpy().copy()
    start = np.array(starts, dtype=np.uint32)
    dep = np.arange(9, dtype=np.uint32)                        # swap-in batch b needs swap-out batch b only
    rows = [tuple(int(x) for x in r) for r in d.tolist()]
    for path_in, taper, bare in ((P.SS_PATH_AUTO, 1, 0), (P.SS_PATH_STAGED, 1, 0), (P.SS_PATH_STAGED, 0, 0),
                                 (P.SS_PATH_AUTO, 1, 1), (P.SS_PATH_STAGED, 1, 1), (P.SS_PATH_STAGED, 0, 1)):
        ctx = make_ctx(P, staging_bytes=h, copy_path=P.SS_PATH_STAGED, copy_path_in=path_in,
                       ring_slot_bytes=1024 * KiB, ring_bytes=2048 * KiB, ring_taper=taper,
                       flags=P.SS_CFG_TIMING | (P.SS_CFG_BARE_RING if bare else 0))
        try:
            P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
            P.ss_load_schedule(ctx, d, start, d, start, dep)
            group_of, group_bytes = P.ss_ring_view(ctx)
            if taper == 1:
                assert group_of.tolist() == [0, 0, 0, -1, 1, 2, -1, 3, 3]
                assert group_bytes.tolist() == [1024 * KiB, 512 * KiB, 768 * KiB, 256 * KiB]
            else:
                # tapered: a swap-out group grows to at most what the groups before it hold (an eighth of a
                # slot, 128 KiB, to begin with; one batch is never split)
                assert group_of.tolist() == [0, 1, 2, -1, 3, 4, -1, 5, 5]
                assert group_bytes.tolist() == [256 * KiB, 512 * KiB, 256 * KiB, 512 * KiB, 768 * KiB, 256 * KiB]
            in_group_of, in_group_bytes = P.ss_ring_view(ctx, 1)
            if path_in == P.SS_PATH_STAGED and taper == 1:   # same slots, same rule: the same groups on the way back
                assert in_group_of.tolist() == group_of.tolist() and in_group_bytes.tolist() == group_bytes.tolist()
            elif path_in == P.SS_PATH_STAGED:
                # tapered: a group takes at most as much as has gone before and at most half of what is still
                # to come (never asked to be less than an eighth of a slot, 128 KiB; one batch is never split):
                # batch 0 travels alone (nothing before it), batches 1 and 2 alone too (256 KiB, then 768 KiB
                # before them: the next batch would not fit), the last two batches (256 KiB to come) one by one
                assert in_group_of.tolist() == [0, 1, 2, -1, 3, 4, -1, 5, 6]
                assert in_group_bytes.tolist() == [256 * KiB, 512 * KiB, 256 * KiB, 512 * KiB, 768 * KiB, 128 * KiB, 128 * KiB]
            else:
                assert (in_group_of == -1).all()
            for order in ([0, 1, 2, 3, 4, 5, 6, 7, 8], [1, 0, 2, 4, 3, 6, 5, 8, 7], [8, 7, 6, 5, 4, 3, 2, 1, 0]):
                arena.copy_(torch.from_numpy(host).cuda())
                P.ss_staging_fill(ctx, 0x11)
                torch.cuda._sleep(2000000)                         # the compute stream lags 2-3 ms behind the calls
                for k, b in enumerate(order):
                    P.ss_swap_out(ctx, b)
                    if k == 1:                                     # release right after the gather
                        P.ss_sync(ctx, P.SS_SYNC_FREE, starts[order[0]])
                for t in range(n):
                    P.ss_sync(ctx, P.SS_SYNC_FREE, t)
                arena.fill_(0x3C)                                  # compute stream: every released block is overwritten
                for b in reversed(order):
                    P.ss_swap_in(ctx, b)
                for t in range(n):
                    P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, t)
                assert P.ss_batch_done(ctx, 0, 3) in (True, False)
                P.ss_sync(ctx, P.SS_SYNC_DRAIN)
                torch.cuda.synchronize()
                staging = np.full(h, 0x11, dtype=np.uint8)
                oracle.swap_out(host, staging, rows)
                assert np.array_equal(P.ss_host_peek(ctx, 0, h), staging), order
                want = np.full(arena_bytes, 0x3C, dtype=np.uint8)
                oracle.swap_in(want, staging, rows)
                assert np.array_equal(arena.cpu().numpy(), want), order
            # a swap-in while the groups of the way out are still open: their gathered part leaves at once
            arena.copy_(torch.from_numpy(host).cuda())
            P.ss_staging_fill(ctx, 0x11)
            for k, b in enumerate([0, 1, 4, 7]):
                P.ss_swap_out(ctx, b)
            P.ss_swap_in(ctx, 1)
            P.ss_swap_in(ctx, 7)
            for b in (2, 3, 5, 6, 8):
                P.ss_swap_out(ctx, b)
            for b in (0, 2, 3, 4, 5, 6, 8):
                P.ss_swap_in(ctx, b)
            P.ss_sync(ctx, P.SS_SYNC_DRAIN)
            torch.cuda.synchronize()
            staging = np.full(h, 0x11, dtype=np.uint8)
            oracle.swap_out(host, staging, rows)
            assert np.array_equal(P.ss_host_peek(ctx, 0, h), staging)
            assert np.array_equal(arena.cpu().numpy(), host)
        finally:
            P.ss_destroy(ctx)
    # guards switch the ring off altogether
    ctx = make_ctx(P, staging_bytes=2 * h + 4096, copy_path=P.SS_PATH_STAGED, guard_bytes=256)
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
        d2 = d.copy()
        d2["host_off"] = 256 + np.cumsum([0] + [(sz + 255) // 256 * 256 + 256 for sz in sizes[:-1]])
        P.ss_load_schedule(ctx, d2, start, d2, start)
        assert (P.ss_ring_view(ctx)[0] == -1).all()
    finally:
        P.ss_destroy(ctx)


@pytest.mark.parametrize("path_in,bare", [(0, 0), (3, 0), (0, 1), (3, 1), (3, 3), (0, 2)])
def test_1p3b_shape_step_through_the_ring_equals_no_swapping(P, torch, path_in, bare):
    """configuration 2, three iterations, every swap-out through the ring (all its sizes are multiples of
    the alignment), blocks poisoned at their release: compute results equal the run without swapping"""
    B = P
    from workloads.harness import SwapRun
    res = []
    for swap in (False, True):
        r = SwapRun(B, torch, 2, swap=swap, bpo=11 << 20, bpo_in=4760000, copy_path=B.SS_PATH_STAGED,
                    copy_path_in=path_in,
                    flags=(B.SS_CFG_POISON_FREE | B.SS_CFG_KEEP_LATE | (B.SS_CFG_BARE_RING if bare & 1 else 0) |
                           (B.SS_CFG_MEMORY_MARKERS if bare & 2 else 0)) if swap else 0)    # bare: 1 = bare ring transfers, 2 = memory markers
        try:
            for _ in range(3):
                r.step() if swap else r.step_noswap()
            res.append((r.compute.result(), B.ss_get_stats(r.ctx), r.bytes_each_way))
        finally:
            r.close()
    (c0, g0), _, _ = res[0]
    (c1, g1), st, moved = res[1]
    assert np.array_equal(c0, c1) and np.array_equal(g0, g1)
    assert st["bytes_out"] == st["bytes_in"] == 3 * moved and st["ring_batches"] == 3 * 120
    assert 0 < st["ring_transfers"] < st["ring_batches"]
    assert (st["ring_batches_in"] > 0) == (path_in == 3) and st["ring_transfers_in"] <= st["ring_batches_in"]


def test_bare_ring_wait_gives_up_after_its_limit_and_the_drain_says_so(P, torch):
    """SS_CFG_BARE_RING with a wait limit of 1 ms and ring transfers of 64 MiB (a little over 1 ms each, queued
    one behind the other): the streams that wait for them give up and go on, every kernel ends normally, and
    SS_SYNC_DRAIN reports SS_E_TIMEOUT; with the default limit the same schedule moves the oracle's bytes.  The
    context stays usable after the error."""
    M = 1 << 20
    nb, sz = 6, 64 * M
    d = np.zeros(nb, dtype=W.DESC_DT)
    for b in range(nb):
        d[b] = (b * sz, b * sz, sz, b, 0)
    start = np.arange(nb + 1, dtype=np.uint32)
    rows = [tuple(int(x) for x in r) for r in d.tolist()]
    arena = random_arena(torch, nb * sz, 77)
    host = arena.cpu().numpy().copy()
    with pytest.raises(P.SsError):
        make_ctx(P, staging_bytes=4096, flag_wait_ms=600001)
    with pytest.raises(P.SsError):
        make_ctx(P, staging_bytes=4096, ring_taper=17)
    for limit in (1, 0):
        ctx = make_ctx(P, staging_bytes=nb * sz, copy_path=P.SS_PATH_STAGED, copy_path_in=P.SS_PATH_STAGED,
                       ring_slot_bytes=sz, ring_bytes=2 * sz, ring_taper=1, flags=P.SS_CFG_BARE_RING, flag_wait_ms=limit)
        try:
            P.ss_bind(ctx, arena.data_ptr(), nb * sz, torch.cuda.current_stream().cuda_stream)
            P.ss_load_schedule(ctx, d, start, d, start, np.arange(nb, dtype=np.uint32))
            for it in range(2):
                arena.copy_(torch.from_numpy(host).cuda())
                for b in range(nb):
                    P.ss_swap_out(ctx, b)
                for t in range(nb):
                    P.ss_sync(ctx, P.SS_SYNC_FREE, t)
                arena.fill_(0x3C)
                for b in reversed(range(nb)):
                    P.ss_swap_in(ctx, b)
                for t in range(nb):
                    P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, t)
                if limit:
                    with pytest.raises(P.SsError) as ei:
                        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
                    assert ei.value.code == P.SS_E_TIMEOUT
                    torch.cuda.synchronize()
                else:
                    P.ss_sync(ctx, P.SS_SYNC_DRAIN)
                    torch.cuda.synchronize()
                    staging = np.zeros(nb * sz, dtype=np.uint8)
                    oracle.swap_out(host, staging, rows)
                    assert np.array_equal(P.ss_host_peek(ctx, 0, nb * sz), staging)
                    assert np.array_equal(arena.cpu().numpy(), host)
        finally:
            P.ss_destroy(ctx)


@pytest.mark.parametrize("seed", range(12))
def test_random_schedules_through_the_rings_both_ways_of_issuing_the_transfers(P, torch, seed):
    """random mixtures of ring-eligible and ragged batches, random slot sizes and counts, tapers 0 / 1 / 4, swap-outs
    in schedule order or shuffled, swap-ins in reverse or shuffled order (each after its swap-out), with events
    behind the ring transfers and bare: staging image and arena equal the oracle's, and both ways of issuing move
    the same bytes"""
    rng = np.random.default_rng(1000 + seed)
    KiB = 1 << 10
    n_batches = int(rng.integers(6, 20))
    sizes, starts = [], [0]
    for b in range(n_batches):
        k = int(rng.integers(1, 4))
        ragged = rng.random() < 0.2
        for _ in range(k):
            sz = int(rng.integers(1, 9)) * 64 * KiB
            if ragged:
                sz += int(rng.integers(1, 200))
            sizes.append(sz)
        starts.append(len(sizes))
    n = len(sizes)
    d = np.zeros(n, dtype=W.DESC_DT)
    off = h = 0
    for i, sz in enumerate(sizes):
        d[i] = (off, h, sz, i, 0)
        off += (sz + 4095) // 4096 * 4096 + 4096
        h += (sz + 255) // 256 * 256
    arena_bytes = off
    arena = random_arena(torch, arena_bytes, 300 + seed)
    host = arena.cpu().numpy().copy()
    start = np.array(starts, dtype=np.uint32)
    dep = np.arange(n_batches, dtype=np.uint32)
    rows = [tuple(int(x) for x in r) for r in d.tolist()]
    slot = int(rng.choice([512, 1024, 2048])) * KiB
    slots = int(rng.integers(2, 5))
    taper = int(rng.choice([0, 1, 4]))
    path_in = int(rng.choice([P.SS_PATH_AUTO, P.SS_PATH_STAGED]))
    order_out = list(range(n_batches))
    if rng.random() < 0.5:
        rng.shuffle(order_out)
    order_in = list(reversed(range(n_batches)))
    if rng.random() < 0.5:
        rng.shuffle(order_in)
    want_staging = np.full(h, 0x11, dtype=np.uint8)
    oracle.swap_out(host, want_staging, rows)
    want_arena = np.full(arena_bytes, 0x3C, dtype=np.uint8)
    oracle.swap_in(want_arena, want_staging, rows)
    stats = []
    for bare in (0, P.SS_CFG_BARE_RING, P.SS_CFG_BARE_RING | P.SS_CFG_MEMORY_MARKERS, P.SS_CFG_MEMORY_MARKERS):
        ctx = make_ctx(P, staging_bytes=h, copy_path=P.SS_PATH_STAGED, copy_path_in=path_in, ring_slot_bytes=slot,
                       ring_bytes=slots * slot, ring_taper=taper, flags=bare)
        try:
            P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
            P.ss_load_schedule(ctx, d, start, d, start, dep)
            for it in range(2):
                arena.copy_(torch.from_numpy(host).cuda())
                P.ss_staging_fill(ctx, 0x11)
                # a compute stream that is 2-3 ms behind the dispatch thread: whatever is not ordered after its
                # marker on that stream runs too early and moves stale bytes
                torch.cuda._sleep(2000000)
                for b in order_out:
                    P.ss_swap_out(ctx, b)
                for t in range(n):
                    P.ss_sync(ctx, P.SS_SYNC_FREE, t)
                torch.cuda._sleep(2000000)
                arena.fill_(0x3C)                      # compute stream: every released block is overwritten
                for b in order_in:
                    P.ss_swap_in(ctx, b)
                for t in range(n):
                    P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, t)
                P.ss_sync(ctx, P.SS_SYNC_DRAIN)
                torch.cuda.synchronize()
                assert np.array_equal(P.ss_host_peek(ctx, 0, h), want_staging), (seed, bare, it)
                assert np.array_equal(arena.cpu().numpy(), want_arena), (seed, bare, it)
            st = P.ss_get_stats(ctx)
            stats.append((st["bytes_out"], st["bytes_in"], st["ring_batches"], st["ring_batches_in"]))
        finally:
            P.ss_destroy(ctx)
    assert all(x == stats[0] for x in stats) and stats[0][0] == 2 * sum(sizes)


def test_batches_outside_the_rings_go_by_copy_kernel_when_ring_transfers_are_bare(P, torch):
    """8 MiB ring slots, batches of 4 and 8 MiB through the rings and batches of 16 MiB that fit no slot: with events
    behind the ring transfers the large ones go by copy engine in both directions (their tensors reach
    engine_min_bytes), with bare ring transfers by copy kernel - a copy-engine transfer behind a kernel that waits
    for a ring transfer would hold up the queue the awaited sequence number travels in.  Same bytes either way."""
    M = 1 << 20
    sizes = [4 * M, 8 * M, 16 * M, 4 * M, 4 * M, 16 * M, 8 * M, 16 * M, 4 * M]
    n = len(sizes)
    d = np.zeros(n, dtype=W.DESC_DT)
    off = 0
    for i, sz in enumerate(sizes):
        d[i] = (off, off, sz, i, 0)
        off += sz
    start = np.arange(n + 1, dtype=np.uint32)
    rows = [tuple(int(x) for x in r) for r in d.tolist()]
    arena = random_arena(torch, off, 41)
    host = arena.cpu().numpy().copy()
    want_staging = np.zeros(off, dtype=np.uint8)
    oracle.swap_out(host, want_staging, rows)
    for bare in (0, 1):
        ctx = make_ctx(P, staging_bytes=off, copy_path=P.SS_PATH_STAGED, copy_path_in=P.SS_PATH_STAGED,
                       ring_slot_bytes=8 * M, ring_bytes=32 * M, ring_taper=1, engine_min_bytes_out=4 * M,
                       flags=P.SS_CFG_BARE_RING if bare else 0)
        try:
            P.ss_bind(ctx, arena.data_ptr(), off, torch.cuda.current_stream().cuda_stream)
            P.ss_load_schedule(ctx, d, start, d, start, np.arange(n, dtype=np.uint32))
            assert [int(g >= 0) for g in P.ss_ring_view(ctx)[0]] == [int(sz <= 8 * M) for sz in sizes]
            for it in range(3):
                arena.copy_(torch.from_numpy(host).cuda())
                for b in range(n):
                    P.ss_swap_out(ctx, b)
                for t in range(n):
                    P.ss_sync(ctx, P.SS_SYNC_FREE, t)
                arena.fill_(0x3C)
                for b in reversed(range(n)):
                    P.ss_swap_in(ctx, b)
                for t in range(n):
                    P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, t)
                P.ss_sync(ctx, P.SS_SYNC_DRAIN)
                torch.cuda.synchronize()
                assert np.array_equal(P.ss_host_peek(ctx, 0, off), want_staging), (bare, it)
                assert np.array_equal(arena.cpu().numpy(), host), (bare, it)
            st = P.ss_get_stats(ctx)
            # (swap-ins are issued in reverse here, so a group whose slot has gone to a later one comes back directly)
            assert st["ring_batches"] == 3 * 6 and 0 < st["ring_batches_in"] <= 3 * 6
            assert st["engine_batches"] == 0 if bare else st["engine_batches"] >= 3 * 6
        finally:
            P.ss_destroy(ctx)


@pytest.mark.parametrize("route", ["auto", "rings with events", "rings bare", "rings bare, memory markers", "auto, memory markers"])
def test_iterations_that_end_without_a_host_wait_equal_no_swapping(P, torch, route):
    """configuration 2, twelve iterations ended with SS_SYNC_ITERATION_END (the host runs on; staging slots and ring
    slots are reused by the next iteration only behind this one's readers, on the device), blocks poisoned at
    their release, then one drain: compute results equal the run without swapping, and the staging area holds the
    last iteration's bytes"""
    B = P
    from workloads.harness import SwapRun
    staged = not route.startswith("auto")
    flags = (B.SS_CFG_POISON_FREE | B.SS_CFG_KEEP_LATE | (B.SS_CFG_BARE_RING if "bare" in route else 0) |
             (B.SS_CFG_MEMORY_MARKERS if "markers" in route else 0))
    res = []
    for swap in (False, True):
        r = SwapRun(B, torch, 2, swap=swap, bpo=11 << 20, bpo_in=4760000,
                    copy_path=B.SS_PATH_STAGED if staged else B.SS_PATH_AUTO,
                    copy_path_in=B.SS_PATH_STAGED if staged else B.SS_PATH_AUTO, flags=flags if swap else 0)
        try:
            if swap:
                r.iteration_end = B.SS_SYNC_ITERATION_END
            for _ in range(12):
                r.step() if swap else r.step_noswap()
            if swap:
                r.drain()
            res.append((r.compute.result(), B.ss_get_stats(r.ctx), r.bytes_each_way))
        finally:
            r.close()
    (c0, g0), _, _ = res[0]
    (c1, g1), st, moved = res[1]
    assert np.array_equal(c0, c1) and np.array_equal(g0, g1)
    assert st["bytes_out"] == st["bytes_in"] == 12 * moved
    assert (st["ring_batches"] > 0) == staged


@pytest.mark.parametrize("path,bare", [(1, 0), (2, 0), (3, 0), (3, 1)])
def test_toy_config_iterations_without_a_host_wait_against_the_oracle(P, torch, path, bare):
    """configuration 1, five iterations ended with SS_SYNC_ITERATION_END and one drain, by copy kernel, by copy
    engine and through rings of two small slots (with events and bare): staging image and arena (with poison over
    released blocks) equal the oracle's after as many iterations; the compute stream lags behind the calls"""
    from paper_2509_11076_amd.executor import run_iteration_dispatch, dispatch_points
    tr = W.build_trace(W.config_shape(1))
    pol = W.config_swap_set(tr, 1)
    idx = pol["ref_op"].astype(np.int64)
    bpo = 64 * 1024
    ap0 = oracle.apply_policy(pol, idx, tr.tensors, bpo)
    swapped = {r[2]: (r[5], r[6]) for r in ap0["resolved"] if not r[3] & 3}
    arena_bytes = place_tensors(tr.tensors, swapped=swapped)
    ora = oracle.apply_policy(pol, idx, tr.tensors, bpo)
    arena = random_arena(torch, arena_bytes, 2509)
    host_arena = arena.cpu().numpy().copy()
    ctx = make_ctx(P, staging_bytes=ora["staging_bytes"], link_bytes_per_op=bpo, copy_path=path, copy_path_in=path,
                   ring_slot_bytes=512 << 10, ring_bytes=1024 << 10,
                   flags=P.SS_CFG_POISON_FREE | (P.SS_CFG_BARE_RING if bare else 0))
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
        lib = P.ss_apply_policy(ctx, pol, idx, tr.tensors)
        assert_applied_equal(lib, P, ctx, ora)
        points = dispatch_points(lib["actions"])
        P.ss_staging_fill(ctx, 0xA5)
        staging = np.full(ora["staging_bytes"], 0xA5, dtype=np.uint8)
        for it in range(5):
            torch.cuda._sleep(1000000)
            run_iteration_dispatch(ctx, tr.n_ops, None, points, end=P.SS_SYNC_ITERATION_END)
            oracle_execute(host_arena, staging, ora, poison=0xDB)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        torch.cuda.synchronize()
        assert np.array_equal(P.ss_host_peek(ctx, 0, ora["staging_bytes"]), staging)
        assert np.array_equal(arena.cpu().numpy(), host_arena)
        st = P.ss_get_stats(ctx)
        assert st["bytes_out"] == st["bytes_in"] == 5 * sum(d[2] for d in ora["descs_out"])
    finally:
        P.ss_destroy(ctx)
