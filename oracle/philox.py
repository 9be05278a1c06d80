"""Philox4x32-10 counter-based random numbers and the dropout masks made from them
(TEST INFRASTRUCTURE ONLY: only tests, the smoke check and the bench's cpu_baseline leg may
import this; it shares no code with the HIP library).

The generator is the published one (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
easy as 1, 2, 3", SC'11, Section 3.3 / Table 2 constants): a 128-bit counter (c0..c3) and a
64-bit key (k0, k1) give four 32-bit words after ten rounds of

    hi0:lo0 = M0 * c0        hi1:lo1 = M1 * c2
    (c0, c1, c2, c3) <- (hi1 ^ c1 ^ k0,  lo1,  hi0 ^ c3 ^ k1,  lo0)

with the key advanced by the Weyl constants (W0, W1) between rounds.

Dropout (the training tasks of Section 6.1 fine-tune with dropout; a recomputed layer must see
the masks of its first forward, which a counter-based generator gives for free): element number
i of a tensor at `site` in iteration `step` reads word i % 4 of the block with

    counter = (low 32 bits of i // 4, high 32 bits of i // 4, site, step),  key = (seed low, seed high)

and is kept when that word >= round(p * 2^32); kept elements are scaled by 1 / (1 - p).  p is a
32-bit float, as at the library's boundary.
"""
from __future__ import annotations

import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK32 = 0xFFFFFFFF

SITE_EMBED = 0


def site_attn_prob(layer: int) -> int:
    return 4 * (layer + 1)


def site_attn_out(layer: int) -> int:
    return 4 * (layer + 1) + 1


def site_ffn_out(layer: int) -> int:
    return 4 * (layer + 1) + 2


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised over the counters (arrays or scalars); returns four uint32 arrays."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & np.uint64(MASK32) for c in (c0, c1, c2, c3))
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0, k1 = int(k0) & MASK32, int(k1) & MASK32
    m = np.uint64(MASK32)
    s32 = np.uint64(32)
    for _ in range(10):
        p0 = np.uint64(M0) * c0                      # 32 x 32 -> 64 bits, exact in uint64
        p1 = np.uint64(M1) * c2
        hi0, lo0 = p0 >> s32, p0 & m
        hi1, lo1 = p1 >> s32, p1 & m
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0, k1 = (k0 + W0) & MASK32, (k1 + W1) & MASK32
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def threshold(p: float) -> int:
    p = float(np.float32(p))
    return min(int(np.floor(p * 4294967296.0 + 0.5)), MASK32)


def words_at(index, seed: int, site: int, step: int) -> np.ndarray:
    """The 32-bit word of every element number in `index` (any shape, uint64)."""
    index = np.asarray(index, dtype=np.uint64)
    block = index >> np.uint64(2)
    w = philox4x32_10(block & np.uint64(MASK32), block >> np.uint64(32), site, step & MASK32,
                      seed & MASK32, (seed >> 32) & MASK32)
    stacked = np.stack(w, axis=-1)                                   # [..., 4]
    which = (index & np.uint64(3)).astype(np.int64)
    return np.take_along_axis(stacked, which[..., None], axis=-1)[..., 0]


def keep_scale(index, p: float, seed: int, site: int, step: int, dtype=np.float64) -> np.ndarray:
    """Multiplier of every element: 0 where dropped, 1 / (1 - p) where kept."""
    p32 = float(np.float32(p))
    keep = words_at(index, seed, site, step) >= np.uint32(threshold(p))
    return keep.astype(dtype) * dtype(1.0 / (1.0 - p32))


def hidden_index(T: int, H: int) -> np.ndarray:
    """Element numbers of a [T, H] activation: row-major."""
    return (np.arange(T, dtype=np.uint64)[:, None] * np.uint64(H) + np.arange(H, dtype=np.uint64)[None, :])


def attn_index(B: int, nh: int, L: int) -> np.ndarray:
    """Element numbers of the [B, nh, L, L] attention probabilities: each row of L keys is padded
    to a multiple of four, so that four neighbouring keys share one block whatever L is."""
    L4 = np.uint64((L + 3) // 4 * 4)
    rows = np.arange(B * nh * L, dtype=np.uint64).reshape(B, nh, L, 1)
    return rows * L4 + np.arange(L, dtype=np.uint64)[None, None, None, :]
