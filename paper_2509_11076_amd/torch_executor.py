"""The swap executor inside a real PyTorch training step (framework glue; no arithmetic of the method).

Sec. 5 of the SmartSwap paper: in the next iteration the swaps of the policy are issued at their
operators, the tensors being recognised by their producing operator and output slot (Sec. 5.1), and a
swapped-out block goes back to the allocator right after the operator the policy names, the compute
stream waiting on the device for the copy (Sec. 5.2).  Here that runs on PyTorch's own tensors:

  * the dispatch hook (libss_torch_hook.so, Detailed mode) numbers the operators and keeps the table of
    the blocks the caching allocator hands out, so a saved tensor's block is known by the operator that
    allocated it and its rank among that operator's allocations;
  * autograd's saved-tensor hooks are the place where the framework hands a tensor over: `pack` keeps a
    policy tensor and returns a handle, `unpack` returns the tensor that came back;
  * between the two, at every hook call, the actions that have become due are issued through libss:
    ss_swap_out_from after operator t_out, ss_sync(FREE) after operator t_free (then the last reference to
    the tensor is dropped and the caching allocator has the block back), ss_swap_in_to from operator t_in
    on, into a block the caching allocator places (torch.empty), ss_sync(WAIT_IN) before the first use.

Only tensors that fill a whole allocator block (contiguous, starting at the block's start, as long as the
block was asked for) are swapped; views into larger blocks stay where they are.
"""
import numpy as np

from . import binding as B
from . import torch_hook as H


class _Handle:
    """what autograd keeps instead of a swapped tensor: the policy item and how this node saw the block (two
    nodes may save the same block under different shapes)"""
    __slots__ = ("item", "dtype", "shape")

    def __init__(self, item, dtype, shape):
        self.item, self.dtype, self.shape = item, dtype, shape


def whole_block(t, blk):
    """a tensor that is all of an allocator block: the block can be given back when the tensor leaves"""
    row, addr = blk
    return (t.is_contiguous() and t.data_ptr() == addr and t.untyped_storage().data_ptr() == addr
            and t.numel() * t.element_size() == int(row["nbytes"]))


class BlockObserver:
    """saved-tensor hooks that change nothing and note, during a profiling iteration, which blocks are held
    by autograd as whole-block tensors (the ones an executor could give back to the allocator)"""

    def __init__(self):
        self.swappable, self.other = set(), set()

    def pack(self, t):
        if t.is_cuda:
            blk = H.ss_hook_block_of(t.untyped_storage().data_ptr())
            if blk is not None:
                (self.swappable if whole_block(t, blk) else self.other).add(int(blk[0]["tensor_id"]))
        return t

    @staticmethod
    def unpack(t):
        return t

    def candidates(self, table):
        """the tensor table with every block that is not held as a whole-block tensor only made ineligible
        (no backward use), so that a policy generator does not pick it"""
        tab = table.copy()
        ok = self.swappable - self.other
        for i in range(len(tab)):
            if int(tab["tensor_id"][i]) not in ok:
                tab["first_bwd_use"][i] = B.SS_NONE_OP
        return tab


PACKED, OUT_ISSUED, FREED, IN_ISSUED, BACK = range(5)


class TorchSwapExecutor:
    """Executes a policy (items with their points t_out, t_free, t_in, t_use in operator indices of the
    hooked sequence) in the iterations that follow.  ctx: a libss context with staging for the policy, no
    arena bound; the dispatch hook must be installed on it in Detailed mode."""

    def __init__(self, torch, ctx, items, descs_out, stream):
        self.torch, self.ctx = torch, ctx
        n = len(items)
        self.items = items
        self.by_identity = {(int(r["ref_op"]), int(r["out_slot"])): k for k, r in enumerate(items)}
        # one batch per tensor each way: batch k is item k
        d = np.zeros(n, dtype=B.DESC_DT)
        host_of = {int(x["tensor_id"]): int(x["host_off"]) for x in descs_out}
        for k, r in enumerate(items):
            d[k] = (0, host_of[int(r["tensor_id"])], int(r["nbytes"]), int(r["tensor_id"]), 0)
        self.descs = d
        start = np.arange(n + 1, dtype=np.uint32)
        B.ss_bind(ctx, None, 0, stream.cuda_stream)
        B.ss_load_schedule(ctx, d, start, d, start, np.arange(n, dtype=np.uint32))
        self.order_out = sorted(range(n), key=lambda k: (int(items["t_out"][k]), k))
        self.order_free = sorted(range(n), key=lambda k: (int(items["t_free"][k]), k))
        self.order_in = sorted(range(n), key=lambda k: (int(items["t_in"][k]), k))
        self.stats = dict(swapped_out=0, freed=0, swapped_in=0, returned_resident=0, bytes_out=0, bytes_in=0,
                          not_seen=0)
        self.capture = None          # optional: callable(item index, tensor) right before its swap-out is issued
        self.before_release = None   # optional: callable(item index, tensor) right before its block is given back
        self.begin_iteration()

    # ---- per iteration -------------------------------------------------------------------------------
    def begin_iteration(self):
        self.state, self.held, self.back = {}, {}, {}
        self.handles = {}            # item -> handles autograd still holds (a tensor saved by two nodes has two)
        self.waited = set()
        self.i_out = self.i_free = self.i_in = 0

    def end_iteration(self):
        """after the optimizer step: joins the swap streams, forgets the iteration"""
        self.stats["not_seen"] += len(self.items) - len(self.state)
        B.ss_sync(self.ctx, B.SS_SYNC_DRAIN)
        self.begin_iteration()

    def hooks(self):
        return self.torch.autograd.graph.saved_tensors_hooks(self.pack, self.unpack)

    # ---- the framework's side: saved-tensor hooks ----------------------------------------------------
    def pack(self, t):
        H.ss_hook_pause(True)        # what the executor itself dispatches is not part of the model's sequence
        try:
            return self._pack(t)
        finally:
            H.ss_hook_pause(False)

    def unpack(self, h):
        # every saved tensor autograd takes back is an occasion to issue what has become due: in the backward
        # pass these calls are the only places the executor is entered
        H.ss_hook_pause(True)
        try:
            self._poll()
            if not isinstance(h, _Handle):
                return h
            return self._unpack(h)
        finally:
            H.ss_hook_pause(False)

    def _pack(self, t):
        self._poll()
        if not t.is_cuda:
            return t
        blk = H.ss_hook_block_of(t.untyped_storage().data_ptr())
        if blk is None or not whole_block(t, blk):
            return t
        k = self.by_identity.get((int(blk[0]["producer_op"]), int(blk[0]["out_slot"])))
        if k is None or int(self.items["nbytes"][k]) != int(blk[0]["nbytes"]):
            return t
        if k not in self.state:
            self.state[k] = PACKED
            self.held[k] = t.detach().reshape(-1).view(self.torch.uint8)      # the block as bytes (same storage)
        self.handles[k] = self.handles.get(k, 0) + 1
        return _Handle(k, t.dtype, tuple(t.shape))

    def _unpack(self, h):
        k = h.item
        st = self.state[k]
        if st in (PACKED, OUT_ISSUED):       # never left (or its block has not been released yet): it is still here
            self.stats["returned_resident"] += 1
            self.back[k] = self.held[k]
            self.state[k] = BACK
        elif st == FREED:                    # the policy's pre-trigger point has not been reached: fetch now
            self._swap_in(k)
        if self.state[k] == IN_ISSUED and k not in self.waited:
            B.ss_sync(self.ctx, B.SS_SYNC_WAIT_IN, int(self.items["tensor_id"][k]))
            self.waited.add(k)
        t = self.back[k].view(h.dtype).view(h.shape)
        self.handles[k] -= 1
        if self.handles[k] == 0:             # the last node that saved it has it now: nothing is kept here
            del self.back[k]
            self.held.pop(k, None)
        return t

    # ---- the executor's side: actions that have become due -------------------------------------------
    def poll(self):
        """issue what is due: `done` operators have been dispatched completely (the one being dispatched
        while a hook runs is not counted)"""
        H.ss_hook_pause(True)
        try:
            self._poll()
        finally:
            H.ss_hook_pause(False)

    def _poll(self):
        done = H.ss_hook_current_op() - 1
        it = self.items
        while self.i_out < len(self.order_out) and int(it["t_out"][self.order_out[self.i_out]]) < done:
            k = self.order_out[self.i_out]
            self.i_out += 1
            if self.state.get(k) == PACKED:
                t = self.held[k]
                if self.capture is not None:
                    self.capture(k, t)
                B.ss_swap_out_from(self.ctx, k, [t.data_ptr()])
                self.state[k] = OUT_ISSUED
                self.stats["swapped_out"] += 1
                self.stats["bytes_out"] += int(it["nbytes"][k])
        while self.i_free < len(self.order_free) and int(it["t_free"][self.order_free[self.i_free]]) < done:
            k = self.order_free[self.i_free]
            self.i_free += 1
            if self.state.get(k) == OUT_ISSUED:
                # the compute stream waits on the device for the copy; from here on the block may be reused
                B.ss_sync(self.ctx, B.SS_SYNC_FREE, int(it["tensor_id"][k]))
                if self.before_release is not None:
                    self.before_release(k, self.held[k])
                del self.held[k]
                self.state[k] = FREED
                self.stats["freed"] += 1
        while self.i_in < len(self.order_in) and int(it["t_in"][self.order_in[self.i_in]]) <= done + 1:
            k = self.order_in[self.i_in]
            if self.state.get(k) in (PACKED, OUT_ISSUED):
                break                        # not released yet: the pointer stays on it
            self.i_in += 1
            if self.state.get(k) == FREED:
                self._swap_in(k)

    def _swap_in(self, k):
        nbytes = int(self.items["nbytes"][k])
        raw = self.torch.empty(nbytes, dtype=self.torch.uint8, device="cuda")     # the caching allocator places the block
        B.ss_swap_in_to(self.ctx, k, [raw.data_ptr()])
        self.back[k] = raw
        self.state[k] = IN_ISSUED
        self.stats["swapped_in"] += 1
        self.stats["bytes_in"] += nbytes


def plan_from_profile(ctx_plan, ops, table, events, base, limit, g_fwd, g_bwd, min_bytes=0, observer=None,
                      phase_bytes_per_op=None):
    """policy for the profiled iteration and its points: the library's generator on the hooked trace, then
    ss_apply_policy (which keeps the generator's release / pre-trigger points when the context was made with
    SS_CFG_POLICY_POINTS).  phase_bytes_per_op: Eq. 1 per phase (link bytes per forward / backward / optimizer
    operator) instead of the one even spread.  Returns (kept items with their points, swap-out descriptors, generator result,
    the application's result, the policy as generated)."""
    tab = observer.candidates(table) if observer is not None else table
    pol, info = B.ss_generate_policy(ctx_plan, ops, tab, events, base, limit, g_fwd, g_bwd, min_bytes=min_bytes,
                                     phase_bytes_per_op=phase_bytes_per_op)
    ap = B.ss_apply_policy(ctx_plan, pol, pol["ref_op"].astype(np.int32), tab, allow_nomem=True)
    res = ap["resolved"]
    kept = res[(res["flags"] & (B.SS_F_UNMATCHED | B.SS_F_ORDER)) == 0]
    return kept, ap["descs_out"], info, ap, pol
