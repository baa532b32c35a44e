"""Synthetic logits: N(0, sigma) by Box-Muller over counter-based uniforms."""
import numpy as np

from .rng import STREAM_LOGITS, draw


def make_logits(seed, B, V, sigma, tag=0):
    """float32 array [B, V]; `tag` selects an independent buffer (e.g. the step)."""
    n = B * V
    n2 = (n + 1) // 2
    base = np.uint64(tag) * np.uint64(1 << 40)
    idx = base + np.arange(2 * n2, dtype=np.uint64)
    u = draw(seed, STREAM_LOGITS, idx)
    # 53-bit uniforms in (0, 1]
    f = ((u >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
    r = np.sqrt(-2.0 * np.log(f[:n2]))
    th = 2.0 * np.pi * f[n2:]
    z = np.concatenate([r * np.cos(th), r * np.sin(th)])[:n]
    return (sigma * z).astype(np.float32).reshape(B, V)


def to_bf16_bits(x32):
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)
