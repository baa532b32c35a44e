"""Counter-based random numbers: value = f(seed, stream, index), no hidden state.

The mixing function is the output stage of SplitMix64 (Steele, Lea, Flood 2014:
add the golden-ratio increment, then two xor-shift-multiply rounds and a final
xor-shift).  A draw chains three applications so that seed, stream and index
each pass through a full avalanche:

    draw(seed, stream, i) = mix(mix(mix(seed) ^ stream) ^ i)

Everything is uint64 with wrap-around, vectorised over the index array, and does
not depend on numpy's own generators (whose streams may change between versions).
"""
import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

STREAM_VOCAB = 1
STREAM_TEMPLATE = 2
STREAM_LOGITS = 3
STREAM_TOKENS = 4


def mix64(x):
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = x + _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def draw(seed, stream, index):
    """uint64 draws for every entry of `index` (any shape)."""
    idx = np.asarray(index, dtype=np.uint64)
    s = mix64(np.uint64(seed))
    s = mix64(s ^ np.uint64(stream))
    return mix64(s ^ idx)


def draw_range(seed, stream, index, n):
    """Draws reduced to [0, n) (plain modulo; n is tiny next to 2**64)."""
    return (draw(seed, stream, index) % np.uint64(n)).astype(np.int64)


class Counter:
    """Sequential convenience wrapper over draw(): each call uses the next index."""

    def __init__(self, seed, stream, start=0):
        self.seed, self.stream, self.i = seed, stream, start

    def u64(self):
        v = int(draw(self.seed, self.stream, np.uint64(self.i)))
        self.i += 1
        return v

    def below(self, n):
        return self.u64() % n

    def between(self, lo, hi):
        """Integer in [lo, hi] inclusive."""
        return lo + self.below(hi - lo + 1)

    def choice(self, seq):
        return seq[self.below(len(seq))]
