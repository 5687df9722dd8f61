"""Pins for the oracle's hash family H (Sec. 3 "Seeding and reproducibility").

The paper names no hash and prints no value; what it requires of H is that
distinct inputs give statistically independent uniform outputs (proof of
Prop. 1).  These tests pin exactly that, plus the constants (re-derived here
by integer square root) and the mixer's structure (an inverse written here,
independently, must undo it).
"""
from math import isqrt

import numpy as np

M64 = (1 << 64) - 1
G64 = ((isqrt(5 << 128) - (1 << 64)) // 2)            # floor(2^64 / phi)
A64 = (isqrt(2 << 128) - (1 << 64)) | 1               # frac(sqrt 2) * 2^64, made odd
B64 = isqrt(3 << 128) - (1 << 64)                     # frac(sqrt 3) * 2^64
G32, A32, B32 = G64 >> 32, A64 >> 32, B64 >> 32


def unmix64(y):
    """Inverse of: x^=x>>32; x*=A; x^=x>>29; x*=B; x^=x>>32."""
    y ^= y >> 32
    y = (y * pow(B64, -1, 1 << 64)) & M64
    y ^= y >> 29
    y ^= y >> 58
    y = (y * pow(A64, -1, 1 << 64)) & M64
    y ^= y >> 32
    return y


def test_constants_are_odd():
    assert A64 & 1 and B64 & 1 and G64 & 1 and G32 & 1 and A32 & 1 and B32 & 1


def test_mix64_is_the_bijection_with_the_derived_constants(orc):
    rng = np.random.default_rng(1)
    xs = [0, 1, M64, 1 << 63] + [int(x) for x in rng.integers(0, 1 << 63, 500)] + \
         [int(x) | (1 << 63) for x in rng.integers(0, 1 << 63, 500)]
    for x in xs:
        assert unmix64(orc.mix64(x)) == x
    assert orc.mix64(0) == 0      # every step fixes zero; callers always xor/add a constant first


def test_combine_structure(orc):
    # combine(h, x) = mix64(h ^ mix64(x + G)): undo the outer mixer, xor h away, undo the inner one
    rng = np.random.default_rng(2)
    for _ in range(300):
        h, x = int(rng.integers(0, 1 << 63)) * 2 + 1, int(rng.integers(0, 1 << 63))
        assert (unmix64(unmix64(orc.combine(h, x)) ^ h) - G64) & M64 == x


def _avalanche(fn, n_in, n_out, trials, rng):
    flips = np.zeros((n_in, n_out))
    for _ in range(trials):
        x = int(rng.integers(0, 1 << 63)) << 1 | int(rng.integers(0, 2))
        x &= (1 << n_in) - 1
        y = fn(x)
        for b in range(n_in):
            d = y ^ fn(x ^ (1 << b))
            flips[b] += [(d >> k) & 1 for k in range(n_out)]
    return flips / trials


def test_mix64_avalanche(orc):
    p = _avalanche(orc.mix64, 64, 64, 1500, np.random.default_rng(3))
    assert 0.43 < p.min() and p.max() < 0.57, (p.min(), p.max())


def test_batch_seed_avalanche_in_every_argument(orc):
    rng = np.random.default_rng(4)
    for which in range(4):
        def fn(x, which=which):
            a = [12345, 3, 7, 11]
            a[which] = x
            return orc.batch_seed(*a)
        nbits = 64 if which == 0 else 32
        p = _avalanche(fn, nbits, 64, 1200, rng)
        assert 0.42 < p.min() and p.max() < 0.58, (which, p.min(), p.max())


def test_key32_avalanche_in_the_neighbour_id(orc):
    rng = np.random.default_rng(5)
    s = int(rng.integers(0, 1 << 63))
    p = _avalanche(lambda u: orc.key32(s, u), 31, 32, 3000, rng)        # node IDs are < 2^31
    assert 0.42 < p.min() and p.max() < 0.58, (p.min(), p.max())


def test_key32_avalanche_in_everything_that_names_the_stream(orc):
    """Prop. 1(b) needs keys of different (s0, w, e, i), hops and frontier nodes
    to be unrelated: flipping any bit of any of them flips every key bit with
    probability about 1/2 (through seed -> hop state -> node state -> key)."""
    rng = np.random.default_rng(6)
    widths = (64, 32, 32, 32, 8, 31)       # s0, w, e, i, hop, v

    def key(a):
        ns = orc.node_state(orc.hop_state(orc.batch_seed(a[0], a[1], a[2], a[3]), a[4]), a[5])
        return orc.key32(ns, a[6])
    trials = 1200
    for which, nbits in enumerate(widths):
        flips = np.zeros((nbits, 32))
        for _ in range(trials):
            a = [int(rng.integers(0, 1 << 62)) & ((1 << wd) - 1) for wd in widths] + [int(rng.integers(0, 1 << 31))]
            y = key(a)
            for b in range(nbits):
                a2 = list(a)
                a2[which] ^= 1 << b
                d = y ^ key(a2)
                flips[b] += [(d >> k) & 1 for k in range(32)]
        p = flips / trials
        assert 0.42 < p.min() and p.max() < 0.58, (which, p.min(), p.max())


def test_key32_uniform_over_consecutive_ids(orc):
    s = orc.node_state(orc.hop_state(orc.batch_seed(0, 0, 0, 0), 0), 17)
    n = 1 << 16
    k = np.array([orc.key32(s, u) for u in range(n)], dtype=np.uint64)
    for shift in (24, 12, 0):           # top, middle and bottom byte
        c = np.bincount(((k >> shift) & 255).astype(np.int64), minlength=256)
        chi2 = ((c - n / 256) ** 2 / (n / 256)).sum()
        assert chi2 < 360, (shift, chi2)          # 255 dof: mean 255, sd 22.6; 360 is +4.6 sd
    # keys of one row are almost always distinct (ties cost bias of order deg / 2^32)
    assert np.unique(k).size > n - 8


def test_streams_are_distinct(orc):
    seen = set()
    for w in range(4):
        for e in range(6):
            seen.add(orc.epoch_state(9, w, e))
            for i in range(40):
                bs = orc.batch_seed(9, w, e, i)
                seen.add(bs)
                for hop in range(3):
                    seen.add(orc.hop_state(bs, hop))
    assert len(seen) == 4 * 6 * (1 + 40 * 4)
    # different base seeds give different streams
    assert orc.batch_seed(0, 0, 0, 0) != orc.batch_seed(1, 0, 0, 0)
