"""CPU ORACLE (test infrastructure, not part of the product path) -- noise generation.

Counter-based random numbers for the PGPE perturbations.  The paper only says that the
algorithm's "ask" generates a population of parameters (Section 4, "Devising New
Algorithms") and that randomness is seeded by keys (Section 4, "Experimenting with More
Tasks"); the generator itself is this build's reading, fixed as follows.

* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
  as 1, 2, 3", SC'11): multipliers 0xD2511F53 / 0xCD9E8D57, Weyl key increments
  0x9E3779B9 / 0xBB67AE85.
* counter = (j, pair k, generation t, stream tag), key = (seed low word, seed high word),
  where j = i >> 2 is the index of the group of four consecutive parameters.
* u32 word x -> uniform u = (2 (x >> 9) + 1) 2^-24 in (0,1); Box-Muller on word pairs:
  (x0,x1) -> z[4j], z[4j+1];  (x2,x3) -> z[4j+2], z[4j+3].

Everything here is evaluated in integer arithmetic (exact) and fp64.
Pins: tests/test_oracle_philox.py (published known-answer vectors, an independent
big-integer implementation, distribution moments).
"""
import numpy as np

PHILOX_M0 = np.uint64(0xD2511F53)
PHILOX_M1 = np.uint64(0xCD9E8D57)
PHILOX_W0 = 0x9E3779B9
PHILOX_W1 = 0xBB67AE85
MASK32 = np.uint64(0xFFFFFFFF)

TAG_NOISE = 0      # PGPE perturbations
TAG_RESET = 1      # task reset states


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox rounds on broadcastable integer arrays; returns four uint32 arrays."""
    c0, c1, c2, c3 = [np.asarray(c, dtype=np.uint64) & MASK32 for c in (c0, c1, c2, c3)]
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = PHILOX_M0 * c0            # 32x32 -> 64 bit products, exact in uint64
        p1 = PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + PHILOX_W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def philox_block(seed, j, k, t, tag):
    """The four output words of counter (j, k, t, tag) under the 64-bit seed."""
    seed = int(seed)
    return philox4x32_10(j, k, t, tag, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)


def u32_to_unit(x):
    """(2 (x >> 9) + 1) / 2^24: an odd multiple of 2^-24, strictly inside (0,1)."""
    x = np.asarray(x, dtype=np.uint32)
    return (2.0 * (x >> np.uint32(9)).astype(np.float64) + 1.0) * 2.0 ** -24


def box_muller(xa, xb):
    """Two standard normals from two u32 words."""
    r = np.sqrt(-2.0 * np.log(u32_to_unit(xa)))
    ang = 2.0 * np.pi * u32_to_unit(xb)
    return r * np.cos(ang), r * np.sin(ang)


def block_normals(seed, j, k, t, tag):
    """Four fp64 standard normals per counter; result shape = broadcast(j,k) + (4,)."""
    x0, x1, x2, x3 = philox_block(seed, j, k, t, tag)
    z0, z1 = box_muller(x0, x1)
    z2, z3 = box_muller(x2, x3)
    return np.stack([z0, z1, z2, z3], axis=-1)


def pair_noise(seed, t, pairs, P, cols=None):
    """z[k, i] for the given pair indices and parameter columns (default: all P), fp64.

    Random access: any (k, i) can be evaluated without generating anything else.
    """
    pairs = np.asarray(pairs, dtype=np.int64).reshape(-1)
    if cols is None:
        nblk = (P + 3) // 4
        z = block_normals(seed, np.arange(nblk)[None, :], pairs[:, None], t, TAG_NOISE)
        return z.reshape(len(pairs), nblk * 4)[:, :P]
    cols = np.asarray(cols, dtype=np.int64).reshape(-1)
    z = block_normals(seed, (cols >> 2)[None, :], pairs[:, None], t, TAG_NOISE)
    return np.take_along_axis(z, np.broadcast_to((cols & 3)[None, :, None], z.shape[:2] + (1,)), axis=2)[..., 0]


def philox_u32_stream(seed, t, k, block0, nblocks, tag):
    """uint32[nblocks*4]: the raw words of counters (block0 .. block0+nblocks-1, k, t, tag)."""
    j = (np.arange(nblocks, dtype=np.uint64) + np.uint64(block0)) & MASK32
    words = philox_block(seed, j, k, t, tag)
    return np.stack(words, axis=-1).reshape(-1)
