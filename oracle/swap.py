"""Byte-level swap round trip (test oracle).

Sec. 1 / Sec. 5.2: a swapped tensor's bytes go from its device block to host
memory after its last forward use and come back, unchanged, into a (possibly
different) device block before its first backward use.  Nothing is compressed
or converted, so the definition is a byte copy per descriptor
(dev_off, host_off, nbytes): nothing outside [host_off, host_off + nbytes) of
the staging area and nothing outside [dev_off, dev_off + nbytes) of the arena
may change.
"""
import numpy as np


class SparseArena:
    """A huge byte arena of which only the blocks ever written are stored.

    Lets the definition below run on a 64 GB arena holding 12 GB of tensors
    without allocating 64 GB.  Blocks are addressed by their exact start.
    """

    def __init__(self):
        self.blocks = {}

    def put(self, off, data):
        self.blocks[int(off)] = np.asarray(data, dtype=np.uint8)

    def read(self, off, n):
        b = self.blocks[int(off)]
        if len(b) < n:
            raise IndexError("read of %d bytes from a %d-byte block" % (n, len(b)))
        return b[:n]

    def write(self, off, data):
        self.blocks[int(off)] = np.array(data, dtype=np.uint8, copy=True)


def _read(arena, off, n):
    if isinstance(arena, SparseArena):
        return arena.read(off, n)
    return arena[off:off + n]


def swap_out(arena, staging, descs):
    """staging[host_off : host_off + nbytes] = arena[dev_off : dev_off + nbytes] for every descriptor."""
    for d in descs:
        dev_off, host_off, n = int(d[0]), int(d[1]), int(d[2])
        staging[host_off:host_off + n] = _read(arena, dev_off, n)


def swap_in(arena, staging, descs):
    """arena[dev_off : dev_off + nbytes] = staging[host_off : host_off + nbytes] for every descriptor."""
    for d in descs:
        dev_off, host_off, n = int(d[0]), int(d[1]), int(d[2])
        if isinstance(arena, SparseArena):
            arena.write(dev_off, staging[host_off:host_off + n])
        else:
            arena[dev_off:dev_off + n] = staging[host_off:host_off + n]
