"""Pins for the oracle's counter-based generator (CPU only)."""
import numpy as np
import pytest

from oracle import philox as ph


def test_generic_w64_matches_numpy_library():
    # numpy.random.Philox is Philox4x64-10 and advances the counter before each block.
    rng = np.random.default_rng(7)
    for _ in range(20):
        key = [int(k) for k in rng.integers(0, 2**63, size=2)]
        ctr = [int(c) for c in rng.integers(0, 2**63, size=4)]
        bg = np.random.Philox(key=key, counter=ctr)
        raw = [int(r) for r in bg.random_raw(8)]
        for blk in range(2):
            c = list(ctr)
            c[0] += blk + 1
            got = ph.philox_generic(c, key, 64, ph.PHILOX_M4x64, ph.PHILOX_W64, 10)
            assert list(got) == raw[4 * blk:4 * blk + 4]


def test_generic_single_round_by_hand():
    # one round, tiny word width, worked by hand from the definition:
    # W=8, M=(3,5), c=(10,20,30,40), k=(1,2):
    # p0=3*10=30 -> hi 0 lo 30 ; p1=5*30=150 -> hi 0 lo 150
    # out = (hi1^c1^k0, lo1, hi0^c3^k1, lo0) = (0^20^1, 150, 0^40^2, 30)
    assert ph.philox_generic((10, 20, 30, 40), (1, 2), 8, (3, 5), (7, 9), rounds=1) == (21, 150, 42, 30)
    # second round bumps the key by the Weyl constants first: k=(8,11)
    # c=(21,150,42,30): p0=63 -> (0,63); p1=210 -> (0,210)
    # out = (0^150^8, 210, 0^30^11, 63)
    assert ph.philox_generic((10, 20, 30, 40), (1, 2), 8, (3, 5), (7, 9), rounds=2) == (158, 210, 21, 63)
    # with carries into the high half: W=8, M0=200, c0=100 -> 20000 = 0x4E20 -> hi 78 lo 32
    assert ph.philox_generic((100, 0, 0, 0), (0, 0), 8, (200, 5), (7, 9), rounds=1) == (0, 0, 78, 32)


def test_vectorised_4x32_matches_generic():
    rng = np.random.default_rng(11)
    n = 300
    c = rng.integers(0, 2**32, size=(4, n), dtype=np.uint64)
    k = [int(t) for t in rng.integers(0, 2**32, size=2, dtype=np.uint64)]
    out = ph.philox4x32_10(c[0], c[1], c[2], c[3], k[0], k[1])
    for i in range(n):
        ref = ph.philox_generic([int(c[j, i]) for j in range(4)], k, 32, ph.PHILOX_M4x32, ph.PHILOX_W32, 10)
        assert tuple(int(o[i]) for o in out) == ref
    # extreme words
    ext = ph.philox4x32_10(0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF)
    ref = ph.philox_generic([0xFFFFFFFF] * 4, [0xFFFFFFFF] * 2, 32, ph.PHILOX_M4x32, ph.PHILOX_W32, 10)
    assert tuple(int(o) for o in ext) == ref


def test_keep_mask_indexing_matches_definition():
    # element idx uses block idx>>3, word (idx>>1)&3, half idx&1 (0 = low 16 bits), with
    # (step_hi, site|layer<<8, step_lo) in the counter
    seed, layer, site, step, p = 0x123456789ABCDEF, 5, 2, (3 << 32) | 17, 0.3
    n = 43
    keep = ph.dropout_keep(seed, layer, site, step, n, p)
    thr = int(np.floor(0.3 * 2**16))
    for idx in (0, 1, 2, 3, 4, 7, 8, 9, 21, 22, 39, 40, 42):
        r = ph.philox_generic((idx >> 3, 3, site | (layer << 8), 17),
                              (seed & 0xFFFFFFFF, seed >> 32), 32, ph.PHILOX_M4x32, ph.PHILOX_W32, 10)
        word = r[(idx >> 1) & 3]
        bits = (word >> 16) if (idx & 1) else (word & 0xFFFF)
        assert bool(keep[idx]) == (bits >= thr)


def test_threshold_and_p_zero():
    assert ph.dropout_threshold(0.1) == 6553
    assert ph.dropout_threshold(0.5) == 32768
    assert ph.dropout_threshold(0.0) == 0
    assert ph.dropout_keep(1, 0, 1, 0, 1000, 0.0).all()
    with pytest.raises(ValueError):
        ph.dropout_threshold(1.0)


def test_halves_of_a_word_are_used_independently():
    # low and high halves of the same output word decide neighbouring elements: their agreement
    # rate is that of independent draws
    n, p = 1 << 20, 0.3
    a = ph.dropout_keep(7, 0, 3, 5, n, p)
    indep = (1 - p) ** 2 + p ** 2
    assert abs((a[0::2] == a[1::2]).mean() - indep) < 5 * np.sqrt(indep * (1 - indep) / (n // 2))


def test_keep_fraction_and_decorrelation():
    n, p = 1 << 20, 0.1
    a = ph.dropout_keep(99, 0, 1, 1, n, p)
    sigma = np.sqrt(p * (1 - p) / n)
    assert abs(a.mean() - (1 - p)) < 5 * sigma
    # a prefix of a longer mask is the shorter mask (pure function of the index)
    assert np.array_equal(a[:1001], ph.dropout_keep(99, 0, 1, 1, 1001, p))
    # other site / step / layer / seed: agreement rate consistent with independence
    indep = (1 - p) ** 2 + p ** 2
    s_ind = np.sqrt(indep * (1 - indep) / n)
    for other in (ph.dropout_keep(99, 0, 2, 1, n, p), ph.dropout_keep(99, 0, 1, 2, n, p),
                  ph.dropout_keep(99, 1, 1, 1, n, p), ph.dropout_keep(100, 0, 1, 1, n, p)):
        assert abs((a == other).mean() - indep) < 5 * s_ind
    # inverted dropout is unbiased: E[x*keep/(1-p)] = x
    x = np.random.default_rng(0).standard_normal(n) + 3.0
    est = (x * a / (1 - p)).mean()
    assert abs(est - x.mean()) < 5 * np.sqrt((x ** 2).mean() * p / (1 - p) / n)
