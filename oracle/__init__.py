"""CPU oracle of the swap-executor hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct Python/NumPy restatement of what the path
computes, written from the paper (SmartSwap, arXiv 2509.11076).  Only the test
suite, the smoke check and the CPU-baseline leg of the benchmark may import
this package; the product (the HIP library and its binding) never does, and
this package imports nothing from the product.  All results are integers or
bytes, so agreement with the HIP path is exact equality.

What the paper fixes and what is this build's reading of it:

* trace_record    - Sec. 3 (Lightweight / Detailed mode).  Record layout and
                    hash function are this build's choice.
* timeline_scan   - Sec. 3 last paragraph + Sec. 4.2 (memory without/with
                    swaps, memory reduction entries).  Intra-operator event
                    order is this build's reading.  Pinned by the live-set
                    definition, brute force over swap sets and a closed form.
* similarity,
  StageMachine    - Sec. 3, Algo. 1 with m = 2, n = 5 (Sec. 6).  Pinned by a
                    hand-derived stage table and exact threshold cases.
* match_anchors   - Sec. 5.1 names the features only; the algorithm is this
                    build's (there is nothing of the paper's to compare with).
                    Pinned by hand cases, an online-counter formulation, the
                    paper's failure case (inserted operators) and invariants.
* apply_policy,
  link_timing     - Sec. 5 first paragraph, Sec. 4.3 (Eq. 3, swap-in
                    pre-trigger, swap-out completion) at operator granularity
                    with a FIFO link; a stand-in for the paper's logical-layer
                    simulator (this build's; the paper prints no values for it).
                    Pinned by hand-worked cases, the schedule checker (also on
                    random policies) and the live-set definition.
* greedy_policy   - stand-in for Algo. 2 (longest-idle-first until the peak
                    fits; this build's).  Pinned by brute force over all
                    subsets on tiny traces.
* swap_out/in     - Sec. 1, 5.2: bytes leave and return unchanged.
* generate_policy - Sec. 4 (Eq. 1-3, Algo. 2): logical layers, MRL, candidate list, simulator.
                    The paper prints no worked example; pinned by a case worked by hand from
                    its steps, the order Eq. 2 prescribes, invariants and brute force.
* align, align_anchors - longest common subsequence of two operator sequences (textbook dynamic
                    programme) and the canonical alignment read off its table; the matcher's fourth
                    level.  Not in the paper (Sec. 5.1 gives no algorithm); pinned by textbook
                    examples, brute force over all subsequences and closed forms.
"""
from .trace import fnv1a32, make_sig, TraceRecorder
from .timeline import timeline_scan
from .match import similarity, StageMachine, match_anchors, match_sequence, WARMUP, GENPOLICY, STABLE
from .policy import (link_timing, apply_policy, greedy_policy, schedule_check,
                     K_IN, K_WAIT_IN, K_OUT, K_FREE,
                     F_UNMATCHED, F_ORDER, F_LATE, F_RESIZED, F_FORCED, Infeasible)
from .swap import swap_out, swap_in, SparseArena
from .generator import generate_policy, generate_policy_best, logical_layers
from .align import align, align_anchors, lcs_table, LEVEL_ALIGN
from .drive import events_by_op, record_trace, ops_tuples, execute_schedule

# The library's call names for the steps that have a one-to-one counterpart here, so that a parity
# test can address both sides by the same name (recording is TraceRecorder.record; the ordering
# calls of the executor have no arithmetic to restate).
ss_timeline_scan = timeline_scan
ss_match_sequence = match_sequence
ss_apply_policy = apply_policy
ss_greedy_policy = greedy_policy
ss_generate_policy = generate_policy
ss_generate_policy_best = generate_policy_best
ss_align_sequence = align_anchors
ss_swap_out = swap_out
ss_swap_in = swap_in
