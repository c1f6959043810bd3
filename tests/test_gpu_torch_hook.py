"""The PyTorch dispatch hook (Sec. 3: Lightweight / Detailed mode) on a real small training step:
what it records is compared with the oracle's recorder fed from an independent observer
(torch.profiler's own operator list), and its memory trace with PyTorch's allocator statistics."""
import argparse

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2509_11076_amd.binding as B
    import paper_2509_11076_amd.torch_hook as H
    from workloads.torch_model import Trainer
    args = argparse.Namespace(vocab=1000, hidden=128, layers=3, heads=4, seq=64, batch=2)
    tr = Trainer(args)
    for _ in range(3):           # allocator and optimizer state settle
        tr.step()
    torch.cuda.synchronize()
    return torch, B, H, tr


def make_ctx(B):
    cfg = B.ss_config_default()
    cfg.staging_bytes = 4096
    cfg.max_ops = 1 << 16
    cfg.max_events = 1 << 18
    return B.ss_create(cfg)


def test_lightweight_sequence_is_stable_and_tokens_follow_first_seen_order(env):
    torch, B, H, tr = env
    ctx = make_ctx(B)
    tr.hook = H
    try:
        H.ss_hook_install(ctx, H.SS_HOOK_LIGHTWEIGHT)
        seqs = []
        for _ in range(3):
            tr.step()
            ops, ev, bal = B.ss_trace_view(ctx)
            seqs.append(ops.copy())
            assert len(ev) == 0 and bal == 0                   # Lightweight mode records no memory events
        n = len(seqs[0])
        assert n > 300
        for s in seqs[1:]:
            assert np.array_equal(s.view(np.uint8), seqs[0].view(np.uint8))
        ops = seqs[0]
        # dense tokens in first-seen order (the recorder's rule)
        first_seen = []
        for t in ops["op_token"].tolist():
            if t not in first_seen:
                first_seen.append(t)
        assert first_seen == list(range(1, len(first_seen) + 1))
        assert (ops["stack_hash"] == 0).all() and (ops["n_out"] == 0).all()
        # phases as the loop announced them: forward, then backward, then optimizer, contiguous
        ph = (ops["sig"] >> 16).tolist()
        assert ph == sorted(ph) and set(ph) == {0, 1, 2}
        # the stage machine sees identical sequences: WarmUp, WarmUp, GenPolicy, ...
        m = [B.ss_match_sequence(ctx, ops, ops, None, flags=B.SS_MATCH_STEP_STAGE) for _ in range(4)]
        assert all(x["similar"] for x in m) and [x["stage"] for x in m] == [0, 0, 1, 1]
        st = H.ss_hook_get_stats()
        assert st["dropped_ops"] == 0 and st["errors"] == 0
    finally:
        H.ss_hook_remove()
        tr.hook = None
        B.ss_destroy(ctx)
    # removed: nothing is recorded any more and the training step still runs
    before = H.ss_hook_get_stats()["ops"]
    tr.step()
    assert H.ss_hook_get_stats()["ops"] == before


def test_operator_names_equal_what_pytorch_profiler_lists(env):
    """independent observer: torch.profiler's CPU operator events of the same step, in start order;
    the oracle's recorder tokenises those names and must give the hook's token sequence"""
    torch, B, H, tr = env
    from torch.profiler import profile, ProfilerActivity
    ctx = make_ctx(B)
    try:
        tr.hook = H
        H.ss_hook_install(ctx, H.SS_HOOK_LIGHTWEIGHT)
        tr.step()
        hook_ops, _, _ = B.ss_trace_view(ctx)
        H.ss_hook_set_mode(H.SS_HOOK_OFF)
        tr.hook = None
        with profile(activities=[ProfilerActivity.CPU]) as prof:
            tr.step()
        # the profiler also lists two kinds of events that are not operator dispatches (other record
        # scopes): the autograd engine's "evaluate_function" wrappers and the optimizer's annotations
        evs = [e for e in prof.events() if e.device_type.name == "CPU" and
               not e.name.startswith("autograd::engine::evaluate_function") and not e.name.startswith("Optimizer.")]
        evs.sort(key=lambda e: (e.time_range.start, -e.time_range.end))
        names = [e.name for e in evs]
        rec = oracle.TraceRecorder()
        toks = [rec.intern(nm, "", 0, 0, 0)[0] for nm in names]
        assert len(toks) == len(hook_ops)
        # both number names densely in first-seen order, so equal sequences of names <=> equal tokens
        assert toks == hook_ops["op_token"].tolist()
    finally:
        H.ss_hook_remove()
        tr.hook = None
        B.ss_destroy(ctx)


def test_detailed_mode_memory_trace_matches_the_allocator(env):
    torch, B, H, tr = env
    ctx = make_ctx(B)
    tr.hook = H
    try:
        H.ss_hook_install(ctx, H.SS_HOOK_DETAILED)
        tr.step()                                              # Detailed once before measuring
        torch.cuda.synchronize()
        # (the gradients that first step's zero_grad freed came before any operator was recorded:
        # such events have no operator to belong to and are counted as dropped)
        dropped0 = H.ss_hook_get_stats()["dropped_events"]
        stats = []
        for _ in range(2):
            tr.opt.zero_grad(set_to_none=True)                 # frees of last step's gradients happen before
            torch.cuda.synchronize()
            # the allocator reports the sizes asked for; its matching statistic is "requested_bytes"
            base = torch.cuda.memory_stats()["requested_bytes.all.current"]
            torch.cuda.reset_peak_memory_stats()
            tr.step()
            torch.cuda.synchronize()
            ops, ev, bal = B.ss_trace_view(ctx)
            peak_torch = torch.cuda.memory_stats()["requested_bytes.all.peak"]
            end_torch = torch.cuda.memory_stats()["requested_bytes.all.current"]
            stats.append((ops.copy(), ev.copy(), bal, base, peak_torch, end_torch))
        ops, ev, bal, base, peak_torch, end_torch = stats[-1]
        assert len(ev) > 100 and (ev["op_idx"][1:] >= ev["op_idx"][:-1]).all()
        # balance of the iteration = what the allocator holds more than at its start (the gradients)
        assert base + bal == end_torch
        # peak: the library's scan and the oracle's agree with each other and with the allocator's own
        # statistic (the allocator's peak can fall between two events of one operator; the scan takes
        # an operator's allocations before its frees, so it can only be the larger)
        lib = B.ss_timeline_scan(ctx, ev, None, len(ops), base, 1 << 62, want_timeline=True)
        ora = oracle.timeline_scan(ev, None, len(ops), base, 1 << 62)
        assert lib["peak"] == ora["peak"] and np.array_equal(lib["per_op"], ora["per_op"])
        running = base + np.cumsum(ev["delta"])                # exact order of the allocator's calls
        assert int(running.max()) == peak_torch
        assert peak_torch <= lib["peak"] <= peak_torch * 1.05
        # Detailed records: outputs known, forward operators carry a call-stack hash, the same operator
        # called from two places gets two hashes
        fwd = ops[(ops["sig"] >> 16) == 0]
        assert (fwd["stack_hash"] != 0).all()
        assert (ops["n_out"] > 0).sum() > 0.5 * len(ops)
        lin = fwd[fwd["n_out"] > 0]
        assert len(set(lin["stack_hash"].tolist())) > 5
        # two Detailed iterations give the same records; tokens equal those of Lightweight mode
        assert np.array_equal(stats[0][0].view(np.uint8), ops.view(np.uint8))
        H.ss_hook_set_mode(H.SS_HOOK_LIGHTWEIGHT)
        tr.step()
        light, _, _ = B.ss_trace_view(ctx)
        assert np.array_equal(light["op_token"], ops["op_token"])
        assert H.ss_hook_get_stats()["dropped_events"] == dropped0
    finally:
        H.ss_hook_remove()
        tr.hook = None
        B.ss_destroy(ctx)


def test_detailed_mode_tensor_table_feeds_the_policy_generator(env):
    """the trace of a real training step goes through the same generator as the synthetic ones: table
    and events agree with each other, saved activations are found, and the policy generated from them
    equals the oracle's on the same table"""
    torch, B, H, _ = env
    from workloads.torch_model import Trainer
    # activations must outweigh parameters and gradients for swapping to lower the peak at all
    tr = Trainer(argparse.Namespace(vocab=1000, hidden=128, layers=3, heads=4, seq=256, batch=8))
    for _ in range(3):
        tr.step()
    ctx = make_ctx(B)
    tr.hook = H
    try:
        H.ss_hook_install(ctx, H.SS_HOOK_DETAILED)
        tr.step()
        tr.opt.zero_grad(set_to_none=True)
        torch.cuda.synchronize()
        base = torch.cuda.memory_stats()["requested_bytes.all.current"]
        tr.step()
        torch.cuda.synchronize()
        ops, ev, bal = B.ss_trace_view(ctx)
        tab = H.ss_hook_tensor_table()
        n_ops = len(ops)
        # one row per allocation, in allocation order, sizes and operators as in the event list
        allocs = ev[ev["delta"] > 0]
        assert len(tab) == len(allocs) and np.array_equal(tab["tensor_id"], allocs["tensor_id"])
        assert np.array_equal(tab["nbytes"].astype(np.int64), allocs["delta"]) and np.array_equal(tab["alloc_op"], allocs["op_idx"])
        frees = {int(e["tensor_id"]): int(e["op_idx"]) for e in ev[ev["delta"] < 0]}
        for row in tab:
            assert int(row["free_op"]) == frees.get(int(row["tensor_id"]), n_ops - 1)
            assert row["alloc_op"] <= row["free_op"]
        # out slots count up within an operator
        for op in np.unique(tab["producer_op"]):
            assert tab["out_slot"][tab["producer_op"] == op].tolist() == list(range(int((tab["producer_op"] == op).sum())))
        # saved activations: allocated in forward, read again in backward, and all of it in order
        ph = ops["sig"] >> 16
        saved = tab[(tab["last_fwd_use"] != 0xFFFFFFFF) & (tab["first_bwd_use"] != 0xFFFFFFFF)]
        assert len(saved) >= 3 * 6                                   # several per decoder layer
        assert (saved["alloc_op"] <= saved["last_fwd_use"]).all() and (saved["last_fwd_use"] < saved["first_bwd_use"]).all()
        assert (saved["first_bwd_use"] <= saved["free_op"]).all()
        assert (ph[saved["last_fwd_use"]] == 0).all() and (ph[saved["first_bwd_use"]] >= 1).all()
        assert (saved["dtype"] != 0).sum() > 0.8 * len(saved)
        # the generator on the real trace: 3 + 3 logical layers (the model has 3 decoder layers)
        no = B.ss_timeline_scan(ctx, ev, None, n_ops, base, 1 << 62)
        cfg = B.ss_config_default()
        cfg.staging_bytes = 4096
        cfg.link_bytes_per_op = 1 << 20
        g = B.ss_create(cfg)
        feasible = 0
        try:
            for frac in (0.98, 0.95, 0.9, 0.8, 0.6):
                limit = base + int(frac * (no["peak"] - base))
                mem = oracle.timeline_scan(ev, None, n_ops, base, limit)["per_op"]
                try:
                    items, _ = oracle.generate_policy(tab, mem, [int(p) for p in ph], limit, 1 << 20, 3, 3, min_bytes=4096)
                except oracle.generator.Infeasible:
                    with pytest.raises(B.SsError) as e:
                        B.ss_generate_policy(g, ops, tab, ev, base, limit, 3, 3, min_bytes=4096)
                    assert e.value.code == B.SS_E_INFEASIBLE
                    continue
                pol, res = B.ss_generate_policy(g, ops, tab, ev, base, limit, 3, 3, min_bytes=4096)
                assert [tuple(int(x) for x in r) for r in pol.tolist()] == items and len(items) > 0
                assert res["peak_no_swap"] == no["peak"] and res["bytes"] == sum(it[8] for it in items)
                assert res["peak_with_policy"] < no["peak"]
                feasible += 1
        finally:
            B.ss_destroy(g)
        assert feasible >= 1, "peak at operator %d of %d, phase %d" % (no["argpeak_op"], n_ops, int(ph[no["argpeak_op"]]))
    finally:
        H.ss_hook_remove()
        tr.hook = None
        B.ss_destroy(ctx)
