"""Philox4x32-10 counter-based random numbers (oracle side).

Follows the published definition (Salmon, Moraes, Dror, Shaw, "Parallel random
numbers: as easy as 1, 2, 3", SC'11, Section 3.3 and Table 2): a 4x32-bit
counter, a 2x32-bit key, ten rounds.  One round multiplies counter words 0 and
2 by two fixed odd constants, producing 64-bit products; the high halves are
XORed with the *other* odd counter word and a key word, the low halves pass
through, and the four words are permuted.  Between rounds the key words are
advanced by the golden-ratio and sqrt(3)-1 Weyl constants.

PBT uses it wherever the method draws a random number (donor choice and
perturbation factor of Section 4.1.1, mini-batch rows, dropout masks, GAN
latents), with the counter assigned as

    c0 = step index or exploit round        c1 = population member
    c2 = domain tag (below) + sub-stream    c3 = element index

and key = (seed & 0xffffffff, seed >> 32).
"""
import numpy as np

PHILOX_M0 = 0xD2511F53
PHILOX_M1 = 0xCD9E8D57
PHILOX_W0 = 0x9E3779B9
PHILOX_W1 = 0xBB67AE85
MASK32 = 0xFFFFFFFF

# Domain tags (counter word c2).  The GPU library uses the same numbers; they
# are part of the interface, like an opcode table.
DOMAIN_BATCH = 1      # c3 = row of the mini-batch; word 0 -> data-set index
DOMAIN_DONOR = 2      # c3 = 0; word 0 -> position in the top set
DOMAIN_EXPLORE = 3    # c3 = hyperparameter index k; bit 0 of word 0 -> factor
DOMAIN_INIT_W = 4     # c0 = 0, c3 = parameter index / 4; words -> uniform init
DOMAIN_INIT_H = 5     # c0 = 0, c3 = hyperparameter index k; word 0 -> prior
DOMAIN_LATENT = 6     # + sub-stream; c3 = element index / 4 -> N(0,1) pairs
DOMAIN_DROPOUT = 16   # + site id; c3 = element index / 4 -> keep masks


def philox4x32_10(ctr, key):
    """ctr: (..., 4) integers < 2**32; key: (2,) integers < 2**32.
    Returns uint32 array of ctr's shape."""
    c = np.asarray(ctr, dtype=np.uint64)
    assert c.shape[-1] == 4
    c0, c1, c2, c3 = (c[..., 0].copy(), c[..., 1].copy(), c[..., 2].copy(), c[..., 3].copy())
    k0 = np.uint64(int(key[0]) & MASK32)
    k1 = np.uint64(int(key[1]) & MASK32)
    m0 = np.uint64(PHILOX_M0)
    m1 = np.uint64(PHILOX_M1)
    mask = np.uint64(MASK32)
    sh = np.uint64(32)
    for r in range(10):
        p0 = m0 * c0          # 32x32 -> 64 bit, exact in uint64
        p1 = m1 * c2
        hi0, lo0 = p0 >> sh, p0 & mask
        hi1, lo1 = p1 >> sh, p1 & mask
        n0 = hi1 ^ c1 ^ k0
        n1 = lo1
        n2 = hi0 ^ c3 ^ k1
        n3 = lo0
        c0, c1, c2, c3 = n0, n1, n2, n3
        if r != 9:
            k0 = (k0 + np.uint64(PHILOX_W0)) & mask
            k1 = (k1 + np.uint64(PHILOX_W1)) & mask
    out = np.stack([c0, c1, c2, c3], axis=-1)
    return out.astype(np.uint32)


def seed_key(seed):
    seed = int(seed)
    return (seed & MASK32, (seed >> 32) & MASK32)


def words(seed, c0, c1, c2, c3):
    """Four uint32 words for one counter (scalars or broadcastable arrays)."""
    c0, c1, c2, c3 = np.broadcast_arrays(np.asarray(c0, dtype=np.uint64),
                                         np.asarray(c1, dtype=np.uint64),
                                         np.asarray(c2, dtype=np.uint64),
                                         np.asarray(c3, dtype=np.uint64))
    ctr = np.stack([c0 & np.uint64(MASK32), c1, c2, c3], axis=-1)
    return philox4x32_10(ctr, seed_key(seed))


def bounded(x, n):
    """Map uint32 word(s) x to an index in [0, n): floor(x * n / 2**32)."""
    return ((np.asarray(x, dtype=np.uint64) * np.uint64(n)) >> np.uint64(32)).astype(np.int64)


def unit_open(x):
    """Map uint32 word(s) to a float64 in the open interval (0, 1)."""
    return (np.asarray(x, dtype=np.float64) + 0.5) / 4294967296.0


def normal_pairs(x_even, x_odd):
    """Box-Muller: two uint32 words -> two independent N(0,1) float64 values."""
    u1 = unit_open(x_even)
    u2 = unit_open(x_odd)
    r = np.sqrt(-2.0 * np.log(u1))
    return r * np.cos(2.0 * np.pi * u2), r * np.sin(2.0 * np.pi * u2)
