"""Synthetic token-byte vocabularies in CSR form.

Layout of every generated vocabulary (stand-in for a byte-level BPE tokenizer's
table; no tokenizer file is read):
  id 0           the end-of-sequence token (no bytes of its own)
  ids 1..256     the 256 single-byte tokens, byte value id-1
  ids 257..V-1   random byte strings, length drawn from the requested
                 distribution, a fraction built from multi-byte UTF-8 sequences
                 (possibly cut mid code point), the rest printable ASCII
The single-byte block guarantees that any FSM state that accepts some byte has a
non-empty mask.
"""
from dataclasses import dataclass

import numpy as np

from .rng import STREAM_VOCAB, draw

_SLOTS = 64          # draw indices reserved per token: 0 length, 1 class, 2.. bytes
N_RESERVED = 257     # EOS + 256 single bytes


@dataclass
class Vocab:
    V: int
    bytes: np.ndarray      # uint8, concatenated token bytes
    offsets: np.ndarray    # uint64, V+1 entries
    eos_id: int
    lmax: int              # longest token in bytes

    def token(self, t):
        return self.bytes[int(self.offsets[t]):int(self.offsets[t + 1])].tobytes()

    def lengths(self):
        return np.diff(self.offsets.astype(np.int64))


def _geometric_lengths(u, mean, cap):
    # P(L >= k+1) = ((mean-1)/mean)**k, cut at cap; thresholds are exact integers
    # so the result is identical on every platform.
    length = np.ones(u.shape, dtype=np.int64)
    for k in range(1, cap):
        thr = (((mean - 1) ** k) << 64) // (mean ** k)
        length += (u < np.uint64(thr)).astype(np.int64)
    return length


def make_vocab(V, dist, seed=0, utf8_tenths=0):
    """dist = ("uniform", lo, hi) or ("geometric", mean, cap); utf8_tenths in 0..10."""
    if V < N_RESERVED:
        raise ValueError("V must be at least 257")
    n = V - N_RESERVED
    tok = np.arange(N_RESERVED, V, dtype=np.uint64)
    base = tok * np.uint64(_SLOTS)
    u_len = draw(seed, STREAM_VOCAB, base)
    if dist[0] == "uniform":
        lo, hi = dist[1], dist[2]
        length = lo + (u_len % np.uint64(hi - lo + 1)).astype(np.int64)
        cap = hi
    elif dist[0] == "geometric":
        mean, cap = dist[1], dist[2]
        length = _geometric_lengths(u_len, mean, cap)
    else:
        raise ValueError(dist)
    assert cap + 2 <= _SLOTS
    is_utf8 = (draw(seed, STREAM_VOCAB, base + np.uint64(1)) % np.uint64(10)).astype(np.int64) < utf8_tenths

    body = np.zeros((n, cap), dtype=np.uint8)
    cont_left = np.zeros(n, dtype=np.int64)        # continuation bytes still owed
    for j in range(cap):
        r = draw(seed, STREAM_VOCAB, base + np.uint64(2 + j))
        ascii_b = (0x20 + (r % np.uint64(95))).astype(np.uint8)
        # multi-byte: a lead byte opens a 2-, 3- or 4-byte sequence, then continuations
        nbytes = 2 + ((r >> np.uint64(8)) % np.uint64(3)).astype(np.int64)
        lead2 = 0xC2 + ((r >> np.uint64(16)) % np.uint64(30))
        lead3 = 0xE1 + ((r >> np.uint64(16)) % np.uint64(12))
        lead4 = 0xF1 + ((r >> np.uint64(16)) % np.uint64(3))
        lead = np.where(nbytes == 2, lead2, np.where(nbytes == 3, lead3, lead4)).astype(np.uint8)
        cont = (0x80 + ((r >> np.uint64(24)) % np.uint64(64))).astype(np.uint8)
        opening = cont_left == 0
        mb = np.where(opening, lead, cont)
        cont_left = np.where(opening, nbytes - 1, cont_left - 1)
        body[:, j] = np.where(is_utf8, mb, ascii_b)

    lengths = np.concatenate([[0], np.ones(256, dtype=np.int64), length])
    offsets = np.zeros(V + 1, dtype=np.uint64)
    offsets[1:] = np.cumsum(lengths).astype(np.uint64)
    data = np.empty(int(offsets[-1]), dtype=np.uint8)
    data[:256] = np.arange(256, dtype=np.uint8)
    keep = np.arange(cap)[None, :] < length[:, None]
    data[256:] = body[keep]
    return Vocab(V=V, bytes=data, offsets=offsets, eos_id=0, lmax=int(lengths.max()))


def tiny_vocab(alphabet, max_len):
    """Every string over `alphabet` (bytes) of length 1..max_len, plus EOS at id 0."""
    toks = [b""]
    frontier = [b""]
    for _ in range(max_len):
        frontier = [p + bytes([a]) for p in frontier for a in alphabet]
        toks.extend(frontier)
    return from_tokens(toks, eos_id=0)


def from_tokens(tokens, eos_id=0):
    lengths = np.array([len(t) for t in tokens], dtype=np.int64)
    offsets = np.zeros(len(tokens) + 1, dtype=np.uint64)
    offsets[1:] = np.cumsum(lengths).astype(np.uint64)
    data = np.frombuffer(b"".join(tokens), dtype=np.uint8).copy()
    return Vocab(V=len(tokens), bytes=data, offsets=offsets, eos_id=eos_id,
                 lmax=int(lengths.max()) if len(tokens) else 0)
