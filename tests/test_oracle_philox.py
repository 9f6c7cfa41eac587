"""Pins of the oracle's counter-based generator and of the draws built on it."""
import os

import numpy as np

import oracle

KAT = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_known_answer_vectors():
    n = 0
    for line in open(KAT):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n == 3


def _philox_py(ctr, key):
    """Philox4x32-10 written a second time, with Python integers."""
    c = list(ctr); k = list(key)
    M = 0xFFFFFFFF
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & M, (p0 >> 32) ^ c[3] ^ k[1], p0 & M]
        k = [(k[0] + 0x9E3779B9) & M, (k[1] + 0xBB67AE85) & M]
    return c


def test_normals_follow_the_stated_box_muller_mapping():
    seed = 0x1234567890ABCDEF
    for (stream, k, t, grp) in [(0, 0, 0, 0), (1, 3, 17, 5), (2, 7, 4999, 123456), (0, 31, 1, 2**31)]:
        r = _philox_py([grp & 0xFFFFFFFF, stream, k, t], [seed & 0xFFFFFFFF, seed >> 32])
        want = []
        for a, b in ((r[0], r[1]), (r[2], r[3])):
            u1 = ((a >> 9) + 0.5) / 2**23
            u2 = (b >> 8) / 2**24
            rad = np.sqrt(-2 * np.log(u1))
            want += [rad * np.cos(2 * np.pi * u2), rad * np.sin(2 * np.pi * u2)]
        got = oracle.normal4(seed, stream, k, t, grp)
        assert np.array_equal(got, np.array(want, dtype=np.float32))


def test_normal_moments():
    run = oracle.Run(K=1, n=400_000, eta=np.ones(2), model="noise", grad_sigma=1.0, seed=9)
    g, _ = run.grad(0, 0)
    assert abs(g.mean()) < 4 / np.sqrt(g.size)
    assert abs(g.var() - 1) < 0.01
    assert abs((g**3).mean()) < 0.02
    assert abs((g**4).mean() - 3) < 0.05
    assert np.abs(g).max() < 5.8                      # sqrt(-2 ln 2^-24) = 5.77
    # lag-1 and in-group correlations vanish
    assert abs(np.mean(g[:-1] * g[1:])) < 0.01
    assert abs(np.mean(g[0::4] * g[1::4])) < 0.01
    # different workers / iterations give different, uncorrelated draws
    g2, _ = run.grad(0, 1)
    assert abs(np.mean(g * g2)) < 0.01


def test_noise_gradient_is_sigma_times_normal_and_index_keyed():
    idx = np.array([0, 1, 2, 3, 4, 1000, 59_999_999], dtype=np.int64)
    sub = oracle.Run(K=2, n=len(idx), eta=np.ones(2), model="noise", grad_sigma=1e-3, seed=3,
                     p_idx=idx)
    full = oracle.Run(K=2, n=1001, eta=np.ones(2), model="noise", grad_sigma=1e-3, seed=3)
    gs, _ = sub.grad(1, 7)
    gf, _ = full.grad(1, 7)
    assert np.array_equal(gs[:6], gf[[0, 1, 2, 3, 4, 1000]])
    z = oracle.normal4(3, 0, 1, 7, 250)                # element 1000 = group 250, lane 0
    assert gs[5] == float(np.float32(1e-3) * z[0])
