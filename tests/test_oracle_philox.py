"""Pins for the oracle's Philox4x32-10: published known-answer vectors, an
independent big-integer transcription of the definition, and bit balance."""
import os
import numpy as np

from oracle import philox

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answer_vectors():
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        out = philox.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10]
        n += 1
    assert n == 3


def _philox_bigint(ctr, key):
    # Python integers, one counter at a time: mulhilo -> xor -> permute, key bumped
    # between rounds (SC'11 Section 3.3).
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r > 0:
            k = [(k[0] + 0x9E3779B9) % 2**32, (k[1] + 0xBB67AE85) % 2**32]
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 // 2**32) ^ c[1] ^ k[0], p1 % 2**32, (p0 // 2**32) ^ c[3] ^ k[1], p0 % 2**32]
    return c


def test_against_bigint_transcription():
    rng = np.random.default_rng(7)
    ctr = rng.integers(0, 2**32, size=(2000, 4), dtype=np.uint64)
    key = [int(v) for v in rng.integers(0, 2**32, size=2, dtype=np.uint64)]
    got = philox.philox4x32_10(ctr, key)
    for i in range(0, 2000, 7):
        assert [int(v) for v in got[i]] == _philox_bigint([int(v) for v in ctr[i]], key)


def test_words_counter_assignment():
    seed = (0x299f31d0 << 32) | 0xa4093822
    w = philox.words(seed, 0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344)
    assert [int(v) for v in w] == [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]


def test_bit_balance_and_bounded():
    w = philox.words(2017, 3, np.arange(4096), philox.DOMAIN_EXPLORE, 0)
    bits = np.unpackbits(w.view(np.uint8))
    assert abs(bits.mean() - 0.5) < 0.005
    idx = philox.bounded(w[:, 0], 12)
    assert idx.min() == 0 and idx.max() == 11
    counts = np.bincount(idx, minlength=12)
    assert counts.min() > 4096 / 12 * 0.75
    assert philox.bounded(np.uint32(0xFFFFFFFF), 12) == 11 and philox.bounded(np.uint32(0), 12) == 0
    u = philox.unit_open(np.array([0, 0xFFFFFFFF], dtype=np.uint32))
    assert 0.0 < u[0] < u[1] < 1.0


def test_normal_pairs_moments():
    w = philox.words(1, 0, 0, philox.DOMAIN_LATENT, np.arange(20000))
    a, b = philox.normal_pairs(w[:, 0], w[:, 1])
    z = np.concatenate([a, b])
    assert abs(z.mean()) < 0.02 and abs(z.std() - 1.0) < 0.02
    assert abs(np.mean(a * b)) < 0.02
