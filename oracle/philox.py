"""Counter-based random numbers for dropout: Philox-4xW-R (Salmon, Moraes,
Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper that this repository follows only says that dropout needs reserved
random state (Section 3.2.1, dialect-operator attribute example); it fixes no
generator.  Reading taken here: the public Philox4x32-10 generator, so that a
mask is a pure function of (seed, layer, site, step, element index) and the
backward pass can recompute it.

Two implementations live here on purpose:

* ``philox_generic`` - Python integers, any word width W; the W=64 instance is
  pinned in the tests against numpy.random.Philox (a library routine of the
  same algorithm), which fixes the round structure, the hi/lo placement, the
  lane permutation and the key schedule.
* ``philox4x32_10`` - vectorised numpy for the W=32 instance the dropout
  masks use; pinned in the tests against ``philox_generic(W=32)``.
"""
import numpy as np

# Published Philox constants (multipliers and Weyl key increments).
PHILOX_M4x32 = (0xD2511F53, 0xCD9E8D57)
PHILOX_W32 = (0x9E3779B9, 0xBB67AE85)
PHILOX_M4x64 = (0xD2E7470EE14C6C93, 0xCA5A826395121157)
PHILOX_W64 = (0x9E3779B97F4A7C15, 0xBB67AE8584CAA73B)


def philox_generic(counter, key, W, M, WEYL, rounds=10):
    """One Philox-4xW block.  counter: 4 ints, key: 2 ints.  Returns 4 ints.

    Round: (c0,c1,c2,c3) -> (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));
    the key is bumped by the Weyl constants between rounds (not after the last).
    """
    mask = (1 << W) - 1
    c0, c1, c2, c3 = [int(c) & mask for c in counter]
    k0, k1 = [int(k) & mask for k in key]
    for r in range(rounds):
        if r > 0:
            k0 = (k0 + WEYL[0]) & mask
            k1 = (k1 + WEYL[1]) & mask
        p0 = M[0] * c0
        p1 = M[1] * c2
        hi0, lo0 = p0 >> W, p0 & mask
        hi1, lo1 = p1 >> W, p1 & mask
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox4x32-10.  Inputs broadcastable integer arrays (values
    < 2**32).  Returns four uint32 arrays."""
    m32 = np.uint64(0xFFFFFFFF)
    sh = np.uint64(32)
    c0, c1, c2, c3 = [np.asarray(c, dtype=np.uint64) & m32 for c in (c0, c1, c2, c3)]
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = np.uint64(int(k0) & 0xFFFFFFFF)
    k1 = np.uint64(int(k1) & 0xFFFFFFFF)
    M0 = np.uint64(PHILOX_M4x32[0])
    M1 = np.uint64(PHILOX_M4x32[1])
    for r in range(10):
        if r > 0:
            k0 = (k0 + np.uint64(PHILOX_W32[0])) & m32
            k1 = (k1 + np.uint64(PHILOX_W32[1])) & m32
        p0 = M0 * c0          # < 2**64, exact in uint64
        p1 = M1 * c2
        hi0, lo0 = p0 >> sh, p0 & m32
        hi1, lo1 = p1 >> sh, p1 & m32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def dropout_threshold(p):
    """16-bit threshold: element is KEPT iff its 16 random bits are >= threshold,
    so P(drop) = floor(p * 2**16) / 2**16."""
    if not (0.0 <= p < 1.0):
        raise ValueError("dropout p must be in [0, 1)")
    return int(np.floor(float(p) * 65536.0))


def dropout_keep(seed, layer_id, site, step, n, p):
    """Boolean keep-mask for n elements (flat index 0..n-1) of one dropout site.

    Element idx uses block counter (idx>>3, step>>32, site | layer_id<<8, step&0xffffffff)
    under key (seed&0xffffffff, seed>>32) and takes 16 bits of the block: output word
    (idx>>1)&3, its low half for even idx, its high half for odd idx.  (The generator's
    cost is per block, so every output bit that the decision can use is used.)
    """
    if p == 0.0:
        return np.ones(n, dtype=bool)
    if (n + 7) // 8 > 0xFFFFFFFF:
        raise ValueError("site too large for a 32-bit block counter")
    thr = dropout_threshold(p)
    nblk = (n + 7) // 8
    blk = np.arange(nblk, dtype=np.uint64)
    r = philox4x32_10(blk, (int(step) >> 32) & 0xFFFFFFFF,
                      (int(site) & 0xFF) | ((int(layer_id) & 0xFFFFFF) << 8),
                      int(step) & 0xFFFFFFFF,
                      int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)
    words = np.stack(r, axis=1)                               # [block][word]
    halves = np.stack([words & np.uint32(0xFFFF), words >> np.uint32(16)], axis=2)   # [block][word][low, high]
    return halves.reshape(-1)[:n] >= np.uint32(thr)
