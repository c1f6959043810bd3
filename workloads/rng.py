"""Counter-based seeded integer generator (SplitMix64) for the synthetic inputs.

Every random choice in the workload generators comes from this class, so one
integer seed fixes a whole configuration.  Value *bytes* of tensors do not
matter to the swap path (nothing is compressed or inspected), so they are
drawn from the same stream as raw 64-bit words or, on the GPU, from a seeded
torch generator.
"""
import numpy as np

_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15


def _mix(z):
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9 & _M64
    z = (z ^ (z >> 27)) * 0x94D049BB133111EB & _M64
    return z ^ (z >> 31)


class SplitMix64:
    """state advances by a fixed odd constant; output is a bijective mix of it."""

    def __init__(self, seed, stream=0):
        self.state = _mix((int(seed) & _M64) ^ _mix((int(stream) + 1) * _GAMMA & _M64))

    def fork(self, stream):
        return SplitMix64(self.state, stream)

    def next_u64(self):
        self.state = (self.state + _GAMMA) & _M64
        return _mix(self.state)

    def uniform(self):
        """float in [0, 1) with 53 random bits"""
        return (self.next_u64() >> 11) * (1.0 / (1 << 53))

    def randint(self, n):
        """integer in [0, n) (n small against 2**64, so modulo bias is ignored)"""
        return self.next_u64() % int(n)

    def bernoulli(self, p):
        return self.uniform() < p

    # ---- bulk forms (NumPy, same sequence as the scalar forms) --------------
    def u64_array(self, n):
        idx = np.arange(1, n + 1, dtype=np.uint64)
        with np.errstate(over="ignore"):
            z = np.uint64(self.state) + idx * np.uint64(_GAMMA)
            self.state = int(z[-1]) if n else self.state
            z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
            z = z ^ (z >> np.uint64(31))
        return z

    def uniform_array(self, n):
        return (self.u64_array(n) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))

    def permutation(self, n):
        """random permutation of range(n): argsort of n random 64-bit keys"""
        keys = self.u64_array(n)
        return np.argsort(keys, kind="stable").astype(np.int64)

    def bytes(self, n):
        """n pseudo-random bytes"""
        words = self.u64_array((n + 7) // 8)
        return words.view(np.uint8)[:n].copy()
