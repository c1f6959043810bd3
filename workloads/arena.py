"""Device-arena placement for the synthetic traces (harness plumbing, not the method).

The swap executor never allocates device memory: the training framework's
allocator does.  Here that allocator is a deterministic first-fit over
residency intervals, so that blocks released early by a swap policy are really
handed to later tensors (the cross-stream reuse situation of Sec. 5.2).
"""
from dataclasses import dataclass
import bisect
import numpy as np


@dataclass
class ArenaPlan:
    offsets: np.ndarray      # one per interval, bytes from the arena base
    arena_bytes: int         # high-water mark (including guards)


def place_first_fit(start_op, end_op, nbytes, align=256, guard=0, capacity=None, reuse_delay=0):
    """Place intervals [start_op, end_op] (inclusive operator indices) of nbytes each.

    A block released after operator e can be taken by an interval starting at
    e + 1 or later, never by one starting at e.  Lowest-address-first fit;
    every block is preceded and followed by `guard` untouched bytes.  Raises
    MemoryError if `capacity` is given and exceeded.  reuse_delay > 0 keeps a
    released block out of the pool for that many more operators (an allocator
    that does not hand a block straight back costs that much memory and lets
    the producer of the next tensor run without waiting for the block's
    previous owner to have left).
    """
    n = len(start_op)
    start_op = np.asarray(start_op, dtype=np.int64)
    end_op = np.asarray(end_op, dtype=np.int64)
    size = (np.asarray(nbytes, dtype=np.int64) + align - 1) // align * align + 2 * guard
    size = (size + align - 1) // align * align
    order = np.lexsort((np.arange(n), start_op))
    by_end = np.lexsort((np.arange(n), end_op))
    offsets = np.zeros(n, dtype=np.int64)
    free_off = [0]            # sorted starts of free extents
    free_len = [1 << 62]
    high = 0
    rel = 0

    def release(off, ln):
        i = bisect.bisect_left(free_off, off)
        free_off.insert(i, off); free_len.insert(i, ln)
        if i + 1 < len(free_off) and free_off[i] + free_len[i] == free_off[i + 1]:
            free_len[i] += free_len[i + 1]; del free_off[i + 1]; del free_len[i + 1]
        if i > 0 and free_off[i - 1] + free_len[i - 1] == free_off[i]:
            free_len[i - 1] += free_len[i]; del free_off[i]; del free_len[i]

    for k in order:
        t = start_op[k]
        while rel < n and end_op[by_end[rel]] + reuse_delay < t:
            j = by_end[rel]
            release(int(offsets[j]) - guard, int(size[j]))
            rel += 1
        need = int(size[k])
        for i in range(len(free_off)):
            if free_len[i] >= need:
                off = free_off[i]
                if free_len[i] == need:
                    del free_off[i]; del free_len[i]
                else:
                    free_off[i] += need; free_len[i] -= need
                break
        offsets[k] = off + guard
        high = max(high, off + need)
        if capacity is not None and high > capacity:
            raise MemoryError("arena capacity %d exceeded (need %d)" % (capacity, high))
    return ArenaPlan(offsets=offsets.astype(np.uint64), arena_bytes=int(high))


def place_tensors(tensors, swapped=None, align=256, guard=0, capacity=None, reuse_delay=0):
    """Fill dev_off / dev_off_in of a tensor table.

    swapped: optional dict tensor_id -> (t_free, t_in); such a tensor is
    resident over [alloc_op, t_free] at dev_off and over [t_in, free_op] at
    dev_off_in.  Others get dev_off_in = dev_off.  Returns the arena size.
    """
    swapped = swapped or {}
    s, e, b, who = [], [], [], []
    for i, t in enumerate(tensors):
        tid = int(t["tensor_id"])
        if tid in swapped:
            t_free, t_in = swapped[tid]
            s += [int(t["alloc_op"]), int(t_in)]
            e += [int(t_free), int(t["free_op"])]
            b += [int(t["nbytes"])] * 2
            who += [(i, 0), (i, 1)]
        else:
            s.append(int(t["alloc_op"])); e.append(int(t["free_op"]))
            b.append(int(t["nbytes"])); who.append((i, 0))
    plan = place_first_fit(s, e, b, align=align, guard=guard, capacity=capacity, reuse_delay=reuse_delay)
    for (i, part), off in zip(who, plan.offsets):
        if part == 0:
            tensors["dev_off"][i] = off
            tensors["dev_off_in"][i] = off
        else:
            tensors["dev_off_in"][i] = off
    return plan.arena_bytes
