"""GPU parity of the byte path: swap-out (gather-pack into pinned staging), release,
swap-in (scatter-unpack) against the oracle's byte copies, bit for bit; guards around every
staging slot and arena block; both copy paths; ragged sizes; block reuse with poison."""
import numpy as np
import pytest

import oracle
import workloads as W
from workloads.arena import place_tensors
from workloads.rng import SplitMix64
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
    words = (nbytes + 7) // 8
    a = torch.randint(-2**62, 2**62, (words,), dtype=torch.int64, device="cuda", generator=g)
    return a.view(torch.uint8)[:nbytes]


def run_schedule(P, ctx, actions, n_ops):
    from paper_2509_11076_amd.executor import run_iteration
    run_iteration(ctx, n_ops, actions, None)


@pytest.mark.parametrize("path", ["kernel", "engine"])
@pytest.mark.parametrize("bpo", [64 * 1024, INSTANT])
def test_toy_config_round_trip_with_guards_and_poison(P, torch, path, bpo):
    """configuration 1: all layer-0 activations of the 2-layer toy block leave and return"""
    guard = 256
    tr = W.build_trace(W.config_shape(1))
    pol = W.config_swap_set(tr, 1)
    idx = pol["ref_op"].astype(np.int64)
    ap0 = oracle.apply_policy(pol, idx, tr.tensors, bpo, guard=guard)
    swapped = {r[2]: (r[5], r[6]) for r in ap0["resolved"] if not r[3] & (oracle.F_UNMATCHED | oracle.F_ORDER)}
    arena_bytes = place_tensors(tr.tensors, swapped=swapped, guard=guard)
    ora = oracle.apply_policy(pol, idx, tr.tensors, bpo, guard=guard)
    assert oracle.schedule_check(ora, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    arena = random_arena(torch, arena_bytes, 2509)
    host_arena = arena.cpu().numpy().copy()
    ctx = make_ctx(P, staging_bytes=ora["staging_bytes"], link_bytes_per_op=bpo, guard_bytes=guard,
                   copy_path=P.SS_PATH_KERNEL if path == "kernel" else P.SS_PATH_ENGINE,
                   copy_path_in=P.SS_PATH_KERNEL if path == "kernel" else P.SS_PATH_ENGINE,
                   flags=P.SS_CFG_POISON_FREE | P.SS_CFG_TIMING)
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
        lib = P.ss_apply_policy(ctx, pol, idx, tr.tensors)
        assert_applied_equal(lib, P, ctx, ora)
        P.ss_staging_fill(ctx, 0xA5)
        staging = np.full(ora["staging_bytes"], 0xA5, dtype=np.uint8)
        run_schedule(P, ctx, lib["actions"], tr.n_ops)
        torch.cuda.synchronize()
        oracle_execute(host_arena, staging, ora, poison=0xDB)
        # staging image: every slot, and every guard / padding byte
        assert np.array_equal(P.ss_host_peek(ctx, 0, ora["staging_bytes"]), staging)
        # arena: every byte, including the poisoned blocks that nobody refilled
        assert np.array_equal(arena.cpu().numpy(), host_arena)
        st = P.ss_get_stats(ctx)
        assert st["bytes_out"] == st["bytes_in"] == sum(d[2] for d in ora["descs_out"])
        assert (st["kernel_batches"] > 0) == (path == "kernel") and (st["engine_batches"] > 0) == (path == "engine")
        _, span = P.ss_batch_ms(ctx, 0)
        assert span >= 0
    finally:
        P.ss_destroy(ctx)


def test_native_dispatch_equals_the_per_action_loop(P, torch):
    """ss_dispatch issues the schedule's actions operator by operator: the toy configuration run with it
    leaves the same staging image, the same arena (poisoned blocks included) and the same statistics as
    one library call per action; and what it refuses"""
    from paper_2509_11076_amd.executor import run_iteration, run_iteration_dispatch, dispatch_points
    tr = W.build_trace(W.config_shape(1))
    pol = W.config_swap_set(tr, 1)
    idx = pol["ref_op"].astype(np.int64)
    ora = oracle.apply_policy(pol, idx, tr.tensors, 64 * 1024)
    swapped = {r[2]: (r[5], r[6]) for r in ora["resolved"] if not r[3] & 3}
    arena_bytes = place_tensors(tr.tensors, swapped=swapped)
    ora = oracle.apply_policy(pol, idx, tr.tensors, 64 * 1024)
    images = []
    for native in (False, True):
        arena = random_arena(torch, arena_bytes, 2509)
        ctx = make_ctx(P, staging_bytes=ora["staging_bytes"], link_bytes_per_op=64 * 1024, flags=P.SS_CFG_POISON_FREE)
        try:
            with pytest.raises(P.SsError) as e:                     # nothing loaded yet
                P.ss_dispatch(ctx, 0, 0)
            assert e.value.code == P.SS_E_STATE
            P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
            lib = P.ss_apply_policy(ctx, pol, idx, tr.tensors)
            P.ss_staging_fill(ctx, 0xA5)
            if native:
                with pytest.raises(P.SsError) as e:
                    P.ss_dispatch(ctx, 0, 2)
                assert e.value.code == P.SS_E_INVAL
                P.ss_dispatch(ctx, 1 << 30, 1)                      # far beyond the last action: nothing to do
                before, after = dispatch_points(lib["actions"])
                assert before and after and max(before | after) < tr.n_ops
                run_iteration_dispatch(ctx, tr.n_ops, None, (before, after))
            else:
                run_iteration(ctx, tr.n_ops, lib["actions"], None)
            torch.cuda.synchronize()
            st = P.ss_get_stats(ctx)
            images.append((P.ss_host_peek(ctx, 0, ora["staging_bytes"]).copy(), arena.cpu().numpy(),
                           {k: st[k] for k in ("bytes_out", "bytes_in", "kernel_batches", "engine_batches", "free_waits", "in_waits")}))
            if native:                                              # a schedule loaded without actions cannot be dispatched
                os_, is_, dep = P.ss_schedule_view(ctx)
                P.ss_load_schedule(ctx, lib["descs_out"], os_, lib["descs_in"], is_, dep)
                with pytest.raises(P.SsError) as e:
                    P.ss_dispatch(ctx, 0, 1)
                assert e.value.code == P.SS_E_STATE
        finally:
            P.ss_destroy(ctx)
    assert np.array_equal(images[0][0], images[1][0]) and np.array_equal(images[0][1], images[1][1])
    assert images[0][2] == images[1][2] and images[0][2]["bytes_out"] == sum(d[2] for d in ora["descs_out"]) > 0
    host_arena = random_arena(torch, arena_bytes, 2509).cpu().numpy().copy()
    staging = np.full(ora["staging_bytes"], 0xA5, dtype=np.uint8)
    oracle_execute(host_arena, staging, ora, poison=0xDB)
    assert np.array_equal(images[1][0], staging) and np.array_equal(images[1][1], host_arena)


def ragged_schedule(seed, n, arena_bytes, max_bytes):
    """descriptors with every awkward size: 0, 1, 15, 16, 17, chunk-1, chunk, chunk+1, several chunks + tail"""
    rng = SplitMix64(seed, 9)
    special = [0, 1, 2, 15, 16, 17, 31, 255, 256, 257, 65535, 65536, 65537, 131071, 3 * 65536 + 5]
    sizes = [special[i] if i < len(special) else 1 + rng.randint(max_bytes) for i in range(n)]
    descs = np.zeros(n, dtype=W.DESC_DT)
    dev, host = 256, 256
    order = rng.permutation(n)
    dev_offs = np.zeros(n, dtype=np.int64)
    for i in order:                      # arena blocks in a shuffled order, 16-byte aligned, guard gaps
        dev_offs[i] = dev
        dev += (sizes[i] + 15) // 16 * 16 + 16 * (1 + rng.randint(8))
    assert dev <= arena_bytes
    for i in range(n):
        descs[i] = (dev_offs[i], host, sizes[i], i, 0)
        host += (sizes[i] + 15) // 16 * 16 + 16 * (1 + rng.randint(4))
    return descs, host + 256


def ragged_round_trip(P, torch, path, seed=3, n=40, max_bytes=200000, arena_bytes=8 << 20, reverse_out=False, **cfg):
    descs, staging_bytes = ragged_schedule(seed, n, arena_bytes // 2, max_bytes)
    n = len(descs)
    out_start = np.array([0, 0, 7, 7, 20, n, n], dtype=np.uint32)       # batches 0, 2 and 5 are empty
    # swap-in to other blocks (upper half of the arena), in another order and batching
    perm = SplitMix64(8).permutation(n)
    descs_in = descs[perm].copy()
    descs_in["dev_off"] += arena_bytes // 2
    in_start = np.array([0, 13, 13, n], dtype=np.uint32)
    arena = random_arena(torch, arena_bytes, 7)
    host_arena = arena.cpu().numpy().copy()
    ctx = make_ctx(P, staging_bytes=staging_bytes, align=16,
                   copy_path=P.SS_PATH_KERNEL if path == "kernel" else P.SS_PATH_ENGINE,
                   copy_path_in=P.SS_PATH_KERNEL if path == "kernel" else P.SS_PATH_ENGINE, **cfg)
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, 0)
        P.ss_load_schedule(ctx, descs, out_start, descs_in, in_start, None)
        P.ss_staging_fill(ctx, 0x5A)
        # the compute stream (the null stream here) lags 2-3 ms behind the calls: a swap-in that is not ordered
        # after the swap-outs it depends on reads the fill pattern
        torch.cuda._sleep(2000000)
        order = range(len(out_start) - 1)
        for b in (reversed(order) if reverse_out else order):
            P.ss_swap_out(ctx, b)
        for b in range(len(in_start) - 1):
            P.ss_swap_in(ctx, b)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        staging = np.full(staging_bytes, 0x5A, dtype=np.uint8)
        oracle.swap_out(host_arena, staging, descs.tolist())
        oracle.swap_in(host_arena, staging, descs_in.tolist())
        assert np.array_equal(P.ss_host_peek(ctx, 0, staging_bytes), staging)
        assert np.array_equal(arena.cpu().numpy(), host_arena)
        return P.ss_get_stats(ctx)
    finally:
        P.ss_destroy(ctx)


@pytest.mark.parametrize("path", ["kernel", "engine"])
def test_ragged_sizes_empty_batches_and_other_destination(P, torch, path):
    ragged_round_trip(P, torch, path)
    # swap-outs issued against their index order, on one swap-out stream and on three: a swap-in then waits for
    # whatever has been issued, not for "the batches up to the last one it needs"
    ragged_round_trip(P, torch, path, reverse_out=True)
    ragged_round_trip(P, torch, path, reverse_out=True, out_streams=3, in_streams=2)
    # the compute stream's position published through device memory instead of an event (copy-kernel batches only)
    ragged_round_trip(P, torch, path, flags=P.SS_CFG_MEMORY_MARKERS)
    ragged_round_trip(P, torch, path, flags=P.SS_CFG_MEMORY_MARKERS, reverse_out=True, out_streams=3, in_streams=2)


@pytest.mark.parametrize("window", [1, 2, 5])
def test_engine_swap_in_window_bounds_what_is_outstanding(P, torch, window):
    """engine_window_in = w: ss_swap_in waits for the engine batch issued w batches earlier; same bytes, and the
    number of waits is what the three swap-in batches of the schedule give"""
    st = ragged_round_trip(P, torch, "engine", engine_window_in=window)
    assert st["engine_window_waits"] == max(0, 3 - window)
    assert ragged_round_trip(P, torch, "kernel", engine_window_in=window)["engine_window_waits"] == 0


@pytest.mark.parametrize("workgroups", [1, 7, 64, 4096])
def test_descriptor_lookup_in_lds_moves_the_same_bytes(P, torch, workgroups):
    """the form of the copy kernel that keeps the batch's chunk-prefix table in LDS and searches it per chunk:
    ragged sizes (empty tensors among them, which share their successor's first chunk), empty batches,
    batches of one tensor and of many, tensors of up to 40 chunks"""
    ragged_round_trip(P, torch, "kernel", copy_desc_lookup=1, copy_workgroups=workgroups)
    ragged_round_trip(P, torch, "kernel", seed=5, n=60, max_bytes=2500000, arena_bytes=256 << 20,
                      copy_desc_lookup=1, copy_workgroups=workgroups)


@pytest.mark.parametrize("workgroups,workgroups_out,unroll", [(1, 1, 1), (3, 5, 2), (64, 8, 4), (4096, 4096, 8), (0, 0, 0)])
def test_every_launch_shape_within_the_limits_moves_the_same_bytes(P, torch, workgroups, workgroups_out, unroll):
    """grids from one workgroup to the maximum, every unroll depth, tensors of up to 40 chunks in batches
    whose chunk size differs; and once with system-scope ordering events"""
    ragged_round_trip(P, torch, "kernel", seed=5, n=60, max_bytes=2500000, arena_bytes=256 << 20,
                      copy_workgroups=workgroups, copy_workgroups_out=workgroups_out, copy_unroll=unroll)
    if workgroups == 0:
        ragged_round_trip(P, torch, "kernel", seed=6, n=60, max_bytes=300000, arena_bytes=64 << 20,
                          flags=P.SS_CFG_SYSTEM_FENCE)
        # swap streams confined to 16 compute units by a unit mask
        ragged_round_trip(P, torch, "kernel", seed=7, n=60, max_bytes=300000, arena_bytes=64 << 20, copy_cus=16)
        with pytest.raises(P.SsError) as e:
            make_ctx(P, staging_bytes=4096, copy_cus=100000)
        assert e.value.code == P.SS_E_INVAL
        for bad in (dict(copy_workgroups=4097), dict(copy_unroll=9), dict(copy_workgroups_out=5000),
                    dict(copy_desc_lookup=2), dict(ring_taper=17)):
            with pytest.raises(P.SsError) as e:
                make_ctx(P, staging_bytes=4096, **bad)
            assert e.value.code == P.SS_E_INVAL


def test_schedule_validation_and_call_order_errors(P, torch):
    arena = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    ctx = make_ctx(P, staging_bytes=1 << 16)
    try:
        d = np.zeros(2, dtype=W.DESC_DT)
        d[0] = (0, 0, 4096, 0, 0); d[1] = (8192, 4096, 4096, 1, 0)
        one = np.array([0, 2], dtype=np.uint32)
        with pytest.raises(P.SsError) as e:                  # not bound yet
            P.ss_load_schedule(ctx, d, one, d, one)
        assert e.value.code == P.SS_E_STATE
        P.ss_bind(ctx, arena.data_ptr(), 1 << 20, 0)

        def expect(code, dd, start=one):
            with pytest.raises(P.SsError) as e:
                P.ss_load_schedule(ctx, dd, start, dd, start)
            assert e.value.code == code
        bad = d.copy(); bad["dev_off"][1] = (1 << 20) - 100       # runs past the arena
        expect(P.SS_E_INVAL, bad)
        bad = d.copy(); bad["host_off"][1] = (1 << 16) - 2048     # runs past the staging area
        expect(P.SS_E_NOMEM, bad)
        bad = d.copy(); bad["dev_off"][0] = 8                     # not 16-byte aligned
        expect(P.SS_E_INVAL, bad)
        bad = d.copy(); bad["host_off"][1] = 2048                 # staging slots overlap
        expect(P.SS_E_INVAL, bad)
        expect(P.SS_E_INVAL, d, np.array([0, 1], dtype=np.uint32))   # batches do not cover the descriptors
        P.ss_load_schedule(ctx, d, one, d, one)
        for call, arg in ((P.ss_swap_out, 1), (P.ss_swap_in, 5)):
            with pytest.raises(P.SsError) as e:
                call(ctx, arg)
            assert e.value.code == P.SS_E_INVAL
        with pytest.raises(P.SsError) as e:                  # swap-in of data that never left
            P.ss_swap_in(ctx, 0)
        assert e.value.code == P.SS_E_STATE
        with pytest.raises(P.SsError) as e:                  # release before its swap-out was issued
            P.ss_sync(ctx, P.SS_SYNC_FREE, 0)
        assert e.value.code == P.SS_E_STATE
        with pytest.raises(P.SsError) as e:                  # host-side query of a batch not issued yet
            P.ss_batch_done(ctx, 0, 0)
        assert e.value.code == P.SS_E_STATE
        P.ss_swap_out(ctx, 0)
        torch.cuda.synchronize()                             # the null stream; the swap stream is not blocking
        import time
        t_end = time.time() + 10
        while not P.ss_batch_done(ctx, 0, 0) and time.time() < t_end:
            time.sleep(0.001)
        assert P.ss_batch_done(ctx, 0, 0)                    # 8 KiB leave within moments
        with pytest.raises(P.SsError) as e:
            P.ss_batch_done(ctx, 0, 7)
        assert e.value.code == P.SS_E_INVAL
        with pytest.raises(P.SsError) as e:                  # twice in one iteration
            P.ss_swap_out(ctx, 0)
        assert e.value.code == P.SS_E_STATE
        with pytest.raises(P.SsError) as e:                  # unknown tensor
            P.ss_sync(ctx, P.SS_SYNC_FREE, 99)
        assert e.value.code == P.SS_E_INVAL
        P.ss_sync(ctx, P.SS_SYNC_FREE, 1)
        P.ss_swap_in(ctx, 0)
        P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, 0)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        P.ss_swap_out(ctx, 0)                                # next iteration: allowed again
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        st = P.ss_get_stats(ctx)
        assert st["free_waits"] == 1 and st["in_waits"] == 1 and st["bytes_out"] == 2 * 8192
        # swap-outs issued against their index order: the swap-in that needs all three is refused until all three
        # have been issued (in index order the last one needed stands for the others)
        d3 = np.zeros(3, dtype=W.DESC_DT)
        for i in range(3):
            d3[i] = (i * 8192, i * 4096, 4096, i, 0)
        P.ss_load_schedule(ctx, d3, np.arange(4, dtype=np.uint32), d3, np.array([0, 3], dtype=np.uint32),
                           np.array([2], dtype=np.uint32))
        P.ss_swap_out(ctx, 2)
        P.ss_swap_out(ctx, 0)
        with pytest.raises(P.SsError) as e:
            P.ss_swap_in(ctx, 0)
        assert e.value.code == P.SS_E_STATE
        P.ss_swap_out(ctx, 1)
        P.ss_swap_in(ctx, 0)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
    finally:
        P.ss_destroy(ctx)


def test_small_tensor_stress_reduced(P, torch):
    """configuration 5 at 1/10 size: 2,000 tensors of 4 KiB..4 MiB, random placement, two permutations"""
    tr, pol, arena_bytes = W.build_small_tensor_stress(n_swap=2000, n_temp=3000, group=100,
                                                       arena_bytes=4 * 10**9)
    bpo = 256 << 20
    idx = pol["ref_op"].astype(np.int64)
    ora = oracle.apply_policy(pol, idx, tr.tensors, bpo)
    # the last groups to leave are the first to be needed again: a few have no room and are dropped
    assert ora["n_dropped"] <= 20 and len(ora["descs_out"]) >= 1980
    assert oracle.schedule_check(ora, tr.tensors, tr.op_inputs, tr.op_outputs) == []
    arena = random_arena(torch, arena_bytes, 5)
    ctx = make_ctx(P, staging_bytes=ora["staging_bytes"], link_bytes_per_op=bpo, flags=P.SS_CFG_POISON_FREE)
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
        lib = P.ss_apply_policy(ctx, pol, idx, tr.tensors)
        assert_applied_equal(lib, P, ctx, ora)
        sp = oracle.SparseArena()
        before = {}
        for d in ora["descs_out"]:
            blk = arena[d[0]:d[0] + d[2]].cpu().numpy().copy()
            sp.put(d[0], blk); before[d[3]] = blk
        staging = np.zeros(ora["staging_bytes"], dtype=np.uint8)
        P.ss_staging_fill(ctx, 0)
        run_schedule(P, ctx, lib["actions"], tr.n_ops)
        torch.cuda.synchronize()
        oracle.swap_out(sp, staging, ora["descs_out"])
        assert np.array_equal(P.ss_host_peek(ctx, 0, ora["staging_bytes"]), staging)
        oracle.swap_in(sp, staging, ora["descs_in"])
        for d in ora["descs_in"]:                      # every tensor is back, byte for byte
            got = arena[d[0]:d[0] + d[2]].cpu().numpy()
            assert np.array_equal(got, sp.read(d[0], d[2])) and np.array_equal(got, before[d[3]])
    finally:
        P.ss_destroy(ctx)


def test_auto_path_of_the_swap_out_side_follows_the_smallest_batch(P, torch):
    """SS_PATH_AUTO: a schedule whose swap-out batches all reach engine_min_bytes_out goes by copy
    engine as a whole, one with a smaller batch goes by copy kernel as a whole; the bytes are the
    same either way"""
    big = 32 << 20
    arena_bytes = 4 * big
    arena = random_arena(torch, arena_bytes, 5)
    want = arena.clone()
    for sizes, engine_out in (((big, big + 4096), True), ((big, big + 4096, 1 << 20), False)):
        d = np.zeros(len(sizes), dtype=W.DESC_DT)
        off = 0
        for i, n in enumerate(sizes):
            d[i] = (off, off, n, i, 0)
            off += (n + 255) // 256 * 256
        start = np.arange(len(sizes) + 1, dtype=np.uint32)           # one batch per tensor
        ctx = make_ctx(P, staging_bytes=off)
        try:
            P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
            P.ss_load_schedule(ctx, d, start, d, start)
            for b in range(len(sizes)):
                P.ss_swap_out(ctx, b)
            for i in range(len(sizes)):
                P.ss_sync(ctx, P.SS_SYNC_FREE, i)
            arena.zero_()                                            # the blocks are free: overwrite them
            for b in range(len(sizes)):
                P.ss_swap_in(ctx, b)
            for i in range(len(sizes)):
                P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, i)
            P.ss_sync(ctx, P.SS_SYNC_DRAIN)
            torch.cuda.synchronize()
            st = P.ss_get_stats(ctx)
            assert st["engine_batches_out"] == (len(sizes) if engine_out else 0)
            assert st["kernel_batches"] == (0 if engine_out else len(sizes) + 1)   # + the 1 MiB swap-in
            assert st["bytes_out"] == st["bytes_in"] == sum(sizes)
            for i, n in enumerate(sizes):
                o = int(d["dev_off"][i])
                assert torch.equal(arena[o:o + n], want[o:o + n]), i
        finally:
            P.ss_destroy(ctx)
        arena.copy_(want)


def test_link_probe_and_batch_windows(P, torch):
    """ss_bw_probe reports all eight rates of the host link (loose sanity bounds: no figure of merit
    is asserted here); ss_batch_window orders the batches of a direction; argument errors"""
    ctx = make_ctx(P, staging_bytes=8 << 20, flags=P.SS_CFG_TIMING, out_streams=1, in_streams=1)
    try:
        bw = P.ss_bw_probe(ctx, 64 << 20, 3)
        assert set(bw) == {"d2h_gbps", "h2d_gbps", "bidir_d2h_gbps", "bidir_h2d_gbps", "kernel_d2h_gbps",
                           "kernel_h2d_gbps", "kernel_bidir_d2h_gbps", "kernel_bidir_h2d_gbps"}
        assert all(0.5 < v < 500 for v in bw.values()), bw
        for bad in ((1024, 3), (64 << 20, 0), (64 << 20, 1001)):
            with pytest.raises(P.SsError) as e:
                P.ss_bw_probe(ctx, *bad)
            assert e.value.code == P.SS_E_INVAL
        n = 4 << 20
        arena = random_arena(torch, 2 * n, 3)
        want = arena.clone()
        d = np.zeros(2, dtype=W.DESC_DT)
        d[0] = (0, 0, n, 0, 0)
        d[1] = (n, n, n, 1, 0)
        start = np.arange(3, dtype=np.uint32)
        P.ss_bind(ctx, arena.data_ptr(), 2 * n, torch.cuda.current_stream().cuda_stream)
        P.ss_load_schedule(ctx, d, start, d, start)
        for b in range(2):
            P.ss_swap_out(ctx, b)
        for b in range(2):
            P.ss_swap_in(ctx, b)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        torch.cuda.synchronize()
        w = [P.ss_batch_window(ctx, dr, b) for dr in (0, 1) for b in (0, 1)]
        assert w[0][0] == 0.0 and all(s <= e for s, e in w)
        assert w[0][1] <= w[1][0] and w[2][1] <= w[3][0]          # one stream per direction: in order
        assert w[1][1] <= w[2][0]                                  # a swap-in starts after the swap-out it reads
        ms, span = P.ss_batch_ms(ctx, 0, 1)
        assert 0 < ms <= span
        assert P.ss_batch_ms_all(ctx, 0).tolist() == [np.float32(P.ss_batch_ms(ctx, 0, b)[0]) for b in (0, 1)]
        assert len(P.ss_batch_ms_all(ctx, 2)) == 0 and len(P.ss_batch_ms_all(ctx, 3)) == 0     # no ring groups
        with pytest.raises(P.SsError):
            P.ss_batch_ms_all(ctx, 1, capacity=1)
        with pytest.raises(P.SsError):
            P.ss_batch_window(ctx, 0, 2)
        assert torch.equal(arena, want)
    finally:
        P.ss_destroy(ctx)


def test_contexts_alive_together_and_one_after_the_other_move_their_own_bytes(P, torch):
    """swap streams are handed from a destroyed context to the next one; two contexts alive at once get streams of
    their own: interleaved swaps of both, in both copy paths and through the rings, against oracle.swap_out /
    swap_in of the same bytes, then a third context made after the first was destroyed"""
    n, k = 1 << 20, 6

    def setup(seed, path):
        ctx = make_ctx(P, staging_bytes=k * n, copy_path=path, copy_path_in=path, ring_slot_bytes=2 * n, ring_bytes=4 * n)
        arena = random_arena(torch, k * n, seed)
        d = np.zeros(k, dtype=W.DESC_DT)
        for t in range(k):
            d[t] = ((k - 1 - t) * n, t * n, n, t, 0)            # staging order reverses the arena order
        start = np.arange(k + 1, dtype=np.uint32)
        P.ss_bind(ctx, arena.data_ptr(), k * n, torch.cuda.current_stream().cuda_stream)
        P.ss_load_schedule(ctx, d, start, d, start)
        return ctx, arena, d

    def check(ctx, arena, d, before):
        descs = [tuple(int(x) for x in r) for r in d.tolist()]
        staging = np.zeros(k * n, dtype=np.uint8)
        oracle.swap_out(before, staging, descs)
        assert np.array_equal(P.ss_host_peek(ctx, 0, k * n), staging)
        back = np.zeros(k * n, dtype=np.uint8)
        oracle.swap_in(back, staging, descs)
        assert np.array_equal(arena.cpu().numpy(), back)

    a = setup(1, P.SS_PATH_KERNEL)
    b = setup(2, P.SS_PATH_STAGED)
    before = [x[1].cpu().numpy().copy() for x in (a, b)]
    for t in range(k):
        for ctx, _, _ in (a, b):
            P.ss_swap_out(ctx, t)
    for ctx, arena, _ in (a, b):
        for t in range(k):
            P.ss_sync(ctx, P.SS_SYNC_FREE, t)
        arena.zero_()                                           # on the compute stream, after the device-side waits
    for t in range(k):
        for ctx, _, _ in (a, b):
            P.ss_swap_in(ctx, t)
    for ctx, _, _ in (a, b):
        for t in range(k):
            P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, t)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
    torch.cuda.synchronize()
    check(*a, before[0])
    check(*b, before[1])
    P.ss_destroy(a[0])
    c = setup(3, P.SS_PATH_ENGINE)                              # takes over the first context's streams
    try:
        before_c = c[1].cpu().numpy().copy()
        for t in range(k):
            P.ss_swap_out(c[0], t)
        for t in range(k):
            P.ss_sync(c[0], P.SS_SYNC_FREE, t)
        c[1].zero_()
        for t in range(k):
            P.ss_swap_in(c[0], t)
        for t in range(k):
            P.ss_sync(c[0], P.SS_SYNC_WAIT_IN, t)
        P.ss_sync(c[0], P.SS_SYNC_DRAIN)
        torch.cuda.synchronize()
        check(*c, before_c)
        assert P.ss_get_stats(b[0])["ring_batches"] > 0         # the second context went through its rings meanwhile
    finally:
        P.ss_destroy(b[0])
        P.ss_destroy(c[0])


@pytest.mark.timeout(300)
def test_copy_kernel_on_gib_tensors_and_a_batch_above_4_gib(P, torch):
    """the copy kernel itself (both directions forced to it) on tensors of the budgeted configurations'
    sizes in ONE batch of 4.66 GiB: 1 GiB + 15 bytes, 1 GiB, 2 GiB (chunk offsets beyond 32 bits),
    512 MiB - 16, 128 MiB + 1, 32 MiB, at scattered places of a 7 GiB arena; the staging image (with
    guards) and the arena after the return into other blocks equal the oracle's byte copies"""
    G = 1 << 30
    sizes = [G + 15, G, 2 * G, (512 << 20) - 16, (128 << 20) + 1, 32 << 20, 1 << 20]
    guard = 256
    arena_bytes = 7 * G
    arena = random_arena(torch, arena_bytes, 77)
    # scattered, unordered source blocks; the tensors return into the mirror-image order of blocks
    order = [3, 0, 5, 2, 6, 1, 4]
    src_off, off = {}, 4096
    for i in order:
        src_off[i] = off
        off += (sizes[i] + 4095) // 4096 * 4096 + 8192
    assert off <= arena_bytes
    dst_off, off = {}, 4096
    for i in reversed(order):
        dst_off[i] = off
        off += (sizes[i] + 4095) // 4096 * 4096 + 8192
    d_out = np.zeros(len(sizes), dtype=W.DESC_DT)
    d_in = np.zeros(len(sizes), dtype=W.DESC_DT)
    h = guard
    for i, n in enumerate(sizes):
        d_out[i] = (src_off[i], h, n, i, 0)
        d_in[len(sizes) - 1 - i] = (dst_off[i], h, n, i, 0)
        h += (n + 255) // 256 * 256 + guard
    start = np.array([0, len(sizes)], dtype=np.uint32)
    assert sum(sizes) > 4 * G
    host = arena.cpu().numpy().copy()
    ctx = make_ctx(P, staging_bytes=h, copy_path=P.SS_PATH_KERNEL, copy_path_in=P.SS_PATH_KERNEL, guard_bytes=guard)
    try:
        P.ss_bind(ctx, arena.data_ptr(), arena_bytes, torch.cuda.current_stream().cuda_stream)
        P.ss_staging_fill(ctx, 0xA5)
        P.ss_load_schedule(ctx, d_out, start, d_in, start)
        P.ss_swap_out(ctx, 0)
        for i in range(len(sizes)):
            P.ss_sync(ctx, P.SS_SYNC_FREE, i)
        arena.fill_(0x3C)                       # compute stream: the released blocks are overwritten
        P.ss_swap_in(ctx, 0)
        for i in range(len(sizes)):
            P.ss_sync(ctx, P.SS_SYNC_WAIT_IN, i)
        P.ss_sync(ctx, P.SS_SYNC_DRAIN)
        torch.cuda.synchronize()
        staging = np.full(h, 0xA5, dtype=np.uint8)
        oracle.swap_out(host, staging, [tuple(int(x) for x in r) for r in d_out.tolist()])
        assert np.array_equal(P.ss_host_peek(ctx, 0, h), staging)
        host[:] = 0x3C
        oracle.swap_in(host, staging, [tuple(int(x) for x in r) for r in d_in.tolist()])
        assert np.array_equal(arena.cpu().numpy(), host)
        st = P.ss_get_stats(ctx)
        assert st["engine_batches"] == 0 and st["kernel_batches"] == 2
    finally:
        P.ss_destroy(ctx)
