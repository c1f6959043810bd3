"""Small-tensor stress input: many variable-size tensors scattered in a large arena.

Tensors that are "too small" give poor link utilisation when moved one by one
(Sec. 4.2); this input makes that case the whole workload: 20,000 tensors of
4 KiB..4 MiB, mixed fp32/bf16, at random 256-byte-aligned non-overlapping
places of a 64 GB arena, leaving in one random order and returning in another,
inside a memory trace of 100,000 alloc/free events.
"""
import math
import numpy as np

from .layouts import TENSOR_DT, POLICY_DT, NONE_OP, DT_BF16, DT_FP32, DT_SIZE, PH_FWD, PH_BWD
from .rng import SplitMix64
from .transformer import Trace, ModelShape, events_of


def build_small_tensor_stress(n_swap=20000, n_temp=30000, group=100, arena_bytes=64 * 10**9,
                              lo=4096, hi=4 * 1024 * 1024, align=256, seed=2509):
    """Returns (trace, policy_rows, arena_bytes).

    Operators: `nb` forward operators followed by `nb` backward operators,
    nb = ceil(n_swap / group).  Forward operator g produces the g-th group of
    the swap-out order (so one batch leaves after it); backward operator h
    first uses the h-th group of the independent swap-in order.  The n_temp
    temporaries live over random operator ranges and are never swapped.
    """
    rng = SplitMix64(seed, 5)
    nb = (n_swap + group - 1) // group
    n_ops = 2 * nb
    T = n_swap + n_temp

    # sizes: log-uniform in [lo, hi], rounded down to the element size
    u = rng.uniform_array(T)
    raw = np.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))
    is_f32 = rng.u64_array(T) & np.uint64(1)
    dt = np.where(is_f32 == 1, DT_FP32, DT_BF16).astype(np.uint32)
    esz = np.where(is_f32 == 1, 4, 2).astype(np.int64)
    nbytes = np.maximum(esz, (np.rint(raw).astype(np.int64) // esz) * esz)

    tab = np.zeros(T, dtype=TENSOR_DT)
    tab["tensor_id"] = np.arange(T)
    tab["dtype"] = dt
    tab["nbytes"] = nbytes

    perm_out = rng.permutation(n_swap)     # position in swap-out order -> tensor id
    perm_in = rng.permutation(n_swap)      # position in first-backward-use order -> tensor id
    pos_out = np.empty(n_swap, dtype=np.int64); pos_out[perm_out] = np.arange(n_swap)
    pos_in = np.empty(n_swap, dtype=np.int64); pos_in[perm_in] = np.arange(n_swap)
    sw = np.arange(n_swap)
    tab["producer_op"][sw] = pos_out // group
    tab["out_slot"][sw] = pos_out % group
    tab["alloc_op"][sw] = pos_out // group
    tab["last_fwd_use"][sw] = pos_out // group
    tab["first_bwd_use"][sw] = nb + pos_in // group
    extra = (rng.u64_array(n_swap) % np.uint64(8)).astype(np.int64)
    tab["free_op"][sw] = np.minimum(n_ops - 1, nb + pos_in // group + extra)

    # temporaries: alloc at a random operator, freed 0..15 operators later
    tp = np.arange(n_swap, T)
    a = (rng.u64_array(n_temp) % np.uint64(n_ops)).astype(np.int64)
    ln = (rng.u64_array(n_temp) % np.uint64(16)).astype(np.int64)
    f = np.minimum(n_ops - 1, a + ln)
    # temporaries get output slots after the swappable outputs of their operator
    order = np.lexsort((tp, a))
    slot = np.zeros(n_temp, dtype=np.int64)
    base_slot = np.bincount(tab["producer_op"][sw].astype(np.int64), minlength=n_ops)
    run = base_slot.copy()
    for k in order:
        slot[k] = run[a[k]]; run[a[k]] += 1
    tab["producer_op"][tp] = a
    tab["out_slot"][tp] = slot
    tab["alloc_op"][tp] = a
    tab["last_fwd_use"][tp] = np.where(a < nb, np.minimum(f, nb - 1), NONE_OP)
    tab["first_bwd_use"][tp] = NONE_OP
    tab["free_op"][tp] = f

    # random non-overlapping placement: shuffle, then spread the slack as random gaps
    place = rng.permutation(T)
    asz = (nbytes + align - 1) // align * align
    slack_units = (arena_bytes - int(asz.sum())) // align
    if slack_units < 0:
        raise ValueError("arena too small")
    w = rng.uniform_array(T + 1)
    gaps = np.floor(w / w.sum() * slack_units).astype(np.int64) * align
    off = np.zeros(T, dtype=np.int64)
    cur = 0
    for r, k in enumerate(place):
        cur += int(gaps[r])
        off[k] = cur
        cur += int(asz[k])
    assert cur <= arena_bytes
    tab["dev_off"] = off
    tab["dev_off_in"] = off

    shape = ModelShape("stress", 0, 0, 0, 0, 0, 0)
    tr = Trace(shape=shape, seq=0)
    n_out = run
    for i in range(n_ops):
        fwd = i < nb
        tr.op_name.append("stress::produce" if fwd else "stress::consume")
        tr.op_stack.append("stress.fwd" if fwd else "stress.bwd")
        tr.op_dtype.append(DT_BF16)
        tr.op_phase.append(PH_FWD if fwd else PH_BWD)
        tr.op_inputs.append([]); tr.op_outputs.append([None] * int(n_out[i]))
        tr.op_base.append(("s", i)); tr.op_layer.append(-1); tr.op_gemm.append(None)
    for k in range(T):
        tr.op_outputs[int(tab["producer_op"][k])][int(tab["out_slot"][k])] = k
    for k in range(n_swap):
        tr.op_inputs[int(tab["first_bwd_use"][k])].append(k)
    tr.tensor_name = ["t%d" % k for k in range(T)]
    tr.tensor_layer = [-1] * T
    tr.tensors = tab
    tr.events = events_of(tab)

    pol = np.zeros(n_swap, dtype=POLICY_DT)
    ids = perm_out
    pol["ref_op"] = tab["producer_op"][ids]
    pol["out_slot"] = tab["out_slot"][ids]
    pol["tensor_id"] = ids
    pol["nbytes"] = tab["nbytes"][ids]
    return tr, pol, arena_bytes
