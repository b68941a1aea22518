"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
as easy as 1, 2, 3", SC'11), written out with 64-bit integer products.

Used by the sampler so that the random numbers of (seed, sequence, position, vocabulary index)
do not depend on which slot or which step of the engine produced them.
"""
import numpy as np

M0 = np.uint64(0xD2511F53)
M1 = np.uint64(0xCD9E8D57)
W0 = np.uint64(0x9E3779B9)
W1 = np.uint64(0xBB67AE85)
MASK = np.uint64(0xFFFFFFFF)
S32 = np.uint64(32)


def philox4x32_10(counter, key):
    """counter: 4 arrays (broadcastable) of 32-bit words c0..c3; key: 2 words k0, k1.
    Returns 4 uint32 arrays: the 4 output words of the 10-round bijection."""
    c0, c1, c2, c3 = [np.asarray(c, dtype=np.uint64) & MASK for c in counter]
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = np.uint64(int(key[0]) & 0xFFFFFFFF)
    k1 = np.uint64(int(key[1]) & 0xFFFFFFFF)
    for rnd in range(10):
        if rnd > 0:                      # the key is bumped between rounds, 9 times in all
            k0 = (k0 + W0) & MASK
            k1 = (k1 + W1) & MASK
        p0 = M0 * c0                     # 32x32 -> 64 bit products
        p1 = M1 * c2
        hi0, lo0 = p0 >> S32, p0 & MASK
        hi1, lo1 = p1 >> S32, p1 & MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def sampler_bits(seed: int, seq_id: int, position: int, vocab: int) -> np.ndarray:
    """32 random bits for every vocabulary index i of one (sequence, position):
    key = (seed low, seed high); counter = (i // 4, position, seq_id low, seq_id high);
    index i takes output word i % 4."""
    nblk = (vocab + 3) // 4
    blk = np.arange(nblk, dtype=np.uint64)
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    ctr = (blk, np.uint64(position & 0xFFFFFFFF), np.uint64(seq_id & 0xFFFFFFFF),
           np.uint64((seq_id >> 32) & 0xFFFFFFFF))
    words = philox4x32_10(ctr, key)
    return np.stack(words, axis=1).reshape(-1)[:vocab]
