"""Trace recording (test oracle).

Sec. 3: in Lightweight mode every dispatched operator becomes one integer, so
an iteration is an integer sequence; in Detailed mode the operator's name, its
tensors' data type and call stack are kept for later identification, and the
memory in use at each operator is tracked.  Sec. 5.1 requires that later
matching needs integer comparisons only, so every string is reduced to an
integer once, when it is first seen.

This build's layout of one operator record: (op_token, stack_hash, sig, n_out)
 - op_token:   dense id of the operator *name*, 1, 2, 3, ... in first-seen
               order; 0 is reserved for padding.
 - stack_hash: 32-bit FNV-1a of the call-stack string (UTF-8).
 - sig:        dtype code | (n_out & 0xff) << 8 | phase << 16.
 - n_out:      number of output tensors.
"""
import numpy as np

_OP_FIELDS = ("op_token", "stack_hash", "sig", "n_out")


def fnv1a32(data: bytes) -> int:
    """32-bit FNV-1a: start at the offset basis, xor in a byte, multiply by the prime."""
    h = 2166136261
    for b in data:
        h ^= b
        h = (h * 16777619) % (1 << 32)
    return h


def make_sig(dtype: int, n_out: int, phase: int) -> int:
    return (dtype & 0xFF) | ((n_out & 0xFF) << 8) | ((phase & 0xFFFF) << 16)


class TraceRecorder:
    """Intern table + per-iteration append-only trace."""

    def __init__(self):
        self.tokens = {}        # operator name -> token
        self.stacks = {}        # call-stack string -> hash (computed once)
        self.begin()

    def begin(self):
        self.ops = []           # tuples (op_token, stack_hash, sig, n_out)
        self.events = []        # tuples (op_idx, tensor_id, delta)

    def intern(self, name: str, stack: str, dtype: int, n_out: int, phase: int):
        if name not in self.tokens:
            self.tokens[name] = len(self.tokens) + 1
        if stack not in self.stacks:
            self.stacks[stack] = fnv1a32(stack.encode("utf-8"))
        return (self.tokens[name], self.stacks[stack], make_sig(dtype, n_out, phase), n_out)

    def record(self, op, events=()):
        """Append one operator and the alloc/free events it caused.

        Every event must carry the index of the operator being recorded; a
        zero token is refused (it is the padding value).
        """
        if op[0] == 0:
            raise ValueError("token 0 is reserved")
        idx = len(self.ops)
        for (op_idx, tensor_id, delta) in events:
            if op_idx != idx:
                raise ValueError("event for operator %d recorded at operator %d" % (op_idx, idx))
        self.ops.append(tuple(int(x) for x in op))
        self.events.extend((int(a), int(b), int(c)) for (a, b, c) in events)

    def event(self, tensor_id, delta):
        """An alloc/free event that becomes known after its operator was recorded (the allocator
        is called while the operator runs): it belongs to the most recently recorded operator."""
        if not self.ops:
            raise ValueError("no operator recorded yet")
        self.events.append((len(self.ops) - 1, int(tensor_id), int(delta)))

    def amend(self, op_idx, dtype, n_out):
        """Data type and output count of an operator are known when it returns: set them on its
        record; token, call-stack hash and phase stay."""
        tok, stack, sig, _ = self.ops[op_idx]
        self.ops[op_idx] = (tok, stack, make_sig(dtype, n_out, sig >> 16), int(n_out))

    def balance(self):
        """Sum of all deltas of the iteration; 0 for a balanced iteration."""
        return sum(d for (_, _, d) in self.events)

    def ops_array(self):
        a = np.zeros(len(self.ops), dtype=[(f, "<u4") for f in _OP_FIELDS])
        for i, o in enumerate(self.ops):
            a[i] = o
        return a

    def events_array(self):
        a = np.zeros(len(self.events), dtype=[("op_idx", "<u4"), ("tensor_id", "<u4"), ("delta", "<i8")])
        for i, e in enumerate(self.events):
            a[i] = e
        return a
