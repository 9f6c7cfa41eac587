"""Pins of the oracle's learning-rate schedules and QSR scheduler.

Eq. (2), the last-round truncation and the warm-up rule of arXiv 2310.14423,
checked against hand arithmetic and against every communication volume the
paper prints (tests/golden/comm_volume_paper.txt).
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "comm_volume_paper.txt")
N_IMAGENET = 1281167


def _rows():
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        rows.append(dict(id=f[0], epochs=int(f[1]), B=int(f[2]), Tw=int(f[3]), sched=f[4],
                         eta_max=float(f[5]), eta_min=float(f[6]), rule=f[7], coef=float(f[8]),
                         H_base=int(f[9]), pct=float(f[10])))
    return rows


def _table(r):
    """Learning-rate table for one golden row, from the oracle's schedule functions."""
    spe = N_IMAGENET // r["B"]
    T = r["epochs"] * spe
    Tw = r["Tw"]
    if r["sched"] == "cosine":
        return oracle.lr_cosine(T, Tw, r["eta_max"], r["eta_min"]), Tw
    if r["sched"] == "linear":
        return oracle.lr_linear(T, Tw, r["eta_max"], r["eta_min"]), Tw
    if r["sched"] == "pow2cos":
        return oracle.lr_pow2cos(T, Tw, r["eta_max"], r["eta_min"]), Tw
    if r["sched"] == "smith":
        # App. F: the peak until epoch 150 of 300, then halved every 30 epochs
        ms = [e * spe for e in (150, 180, 210, 240, 270)]
        return oracle.lr_step(T, Tw, r["eta_max"], ms, 2.0), Tw
    raise ValueError(r["sched"])


@pytest.mark.parametrize("row", _rows(), ids=lambda r: r["id"])
def test_printed_communication_volume(row):
    eta, Tw = _table(row)
    gamma = 3 if row["rule"] == "cubic" else 2
    H, sync_t = oracle.schedule(eta, Tw, row["H_base"], row["coef"], gamma)
    assert sync_t[-1] == len(eta) and H.sum() == len(eta)
    pct = 100.0 * len(H) / len(eta)
    # the paper prints one decimal
    assert abs(pct - row["pct"]) <= 0.05 + 1e-9, (pct, row["pct"])


def test_eq2_by_hand():
    # App. C.2, caption of the H-schedule figure: H_base=4, alpha=0.0175, eta_max=0.008:
    # (0.0175/0.008)^2 = 4.785...  -> 4
    eta = np.full(1000, 0.008)
    assert oracle.get_H(eta, 0, 0, 4, 0.0175) == 4
    assert oracle.get_H(eta, 0, 0, 2, 0.0175) == 4        # floor term binds, not H_base
    assert oracle.get_H(eta, 0, 0, 8, 0.0175) == 8        # H_base binds
    # (0.25/0.08)^2 = 9.765625 ; (0.25/0.008)^2 = 976.5625
    assert oracle.get_H(np.full(2000, 0.08), 0, 0, 4, 0.25) == 9
    assert oracle.get_H(np.full(2000, 0.008), 0, 0, 4, 0.25) == 976
    assert oracle.get_H(np.full(2000, 0.8), 0, 0, 4, 0.25) == 4
    # exact square: alpha/eta = 2 exactly in binary floating point
    assert oracle.get_H(np.full(100, 0.1), 0, 0, 2, 0.2) == 4
    # general power (Sec. 2) and the cubic rule (App. F): (0.0075/0.001)^3 = 421.875
    assert oracle.get_H(np.full(1000, 0.001), 0, 0, 4, 0.0075, gamma=3) == 421
    assert oracle.get_H(np.full(1000, 0.001), 0, 0, 4, 0.0075, gamma=1) == 7


def test_truncation_forces_sync_at_T():
    eta = np.full(2000, 0.008)
    # 976 > remaining 500 -> H = T - t
    assert oracle.get_H(eta, 0, 1500, 4, 0.25) == 500
    assert oracle.get_H(eta, 0, 1999, 4, 0.25) == 1
    # H_base larger than what is left
    assert oracle.get_H(np.full(10, 0.8), 0, 8, 4, 0.25) == 2
    # eta == 0 (tail of a cosine that reaches 0) and absurdly small eta
    z = np.full(100, 0.0)
    assert oracle.get_H(z, 0, 10, 4, 0.25) == 90
    assert oracle.get_H(np.full(100, 1e-300), 0, 10, 4, 0.25) == 90


def test_warmup_uses_first_post_warmup_round():
    # linear warm-up to 8e-4 over 100 steps, then cosine over T=2000 (ViT-like ratios):
    # every round that starts inside the warm-up takes (alpha/eta_max)^2 = 478.5.. -> 478
    eta = oracle.lr_cosine(2000, 100, 8e-4, 0.0)
    assert eta[0] == 0.0 and eta[100] == 8e-4
    for t in (0, 1, 50, 99):
        assert oracle.get_H(eta, 100, t, 4, 0.0175) == 478
    H, st = oracle.schedule(eta, 100, 4, 0.0175)
    assert H[0] == 478 and st[-1] == 2000


def test_cosine_closed_form_points():
    T, Tw = 1000, 100
    eta = oracle.lr_cosine(T, Tw, 0.5, 0.01)
    assert eta[0] == 0.0
    assert eta[50] == pytest.approx(0.25, rel=1e-15)
    assert eta[Tw] == 0.5                                     # cos(0) = 1
    assert eta[Tw + 450] == pytest.approx(0.255, rel=1e-14)   # midpoint: cos(pi/2) = 0
    assert eta[Tw + 300] == pytest.approx(0.01 + 0.245 * 1.5, rel=1e-14)   # cos(pi/3) = 1/2
    assert eta[-1] > 0.01 and eta[-1] == pytest.approx(
        0.01 + 0.245 * (1 + math.cos(math.pi * 899 / 900)), rel=1e-12)
    assert np.all(np.diff(eta[Tw:]) < 0)


def test_linear_and_pow2cos_closed_form_points():
    eta = oracle.lr_linear(1000, 100, 0.5, 0.1)
    assert eta[0] == 0.0 and eta[100] == 0.5
    assert eta[550] == pytest.approx(0.3, rel=1e-15) and eta[999] == pytest.approx(0.1 + 0.4 / 900, rel=1e-12)
    cos = oracle.lr_cosine(1000, 100, 0.5, 0.0)
    p2 = oracle.lr_pow2cos(1000, 100, 0.5, 0.0)
    assert np.array_equal(p2[:100], cos[:100])                    # warm-up untouched
    assert p2[100] == 0.5 and p2[550] == 0.25                     # cos: 0.5, 0.25
    lg = np.log2(p2[100:])
    assert np.all(lg == np.round(lg))                             # exact powers of two
    assert np.all(np.abs(np.log2(cos[100:]) - lg) <= 0.5 + 1e-12)  # nearest in log scale
    assert np.all(np.diff(p2[100:]) <= 0)


def test_step_schedule_values():
    eta = oracle.lr_step(2000, 0, 0.8, [1000, 1500], 10.0)
    assert eta[0] == 0.8 and eta[999] == 0.8
    assert eta[1000] == 0.08 and eta[1499] == 0.08
    assert eta[1500] == 0.008 and eta[1999] == 0.008


def test_worked_sequences_of_the_five_workloads():
    """H sequences at the benchmark workloads, derived by hand from Eq. (2)."""
    # lsq: cosine 0.1 -> 0, T=256, alpha=0.2, H_base=2
    H, st = oracle.schedule(oracle.lr_cosine(256, 0, 0.1), 0, 2, 0.2)
    assert list(H) == [4] * 14 + [5, 5, 5, 5, 6, 6, 7, 8, 9, 11, 14, 20, 37, 62]
    assert list(st[-5:]) == [123, 137, 157, 194, 256]
    # mlp: 0.8 / 0.08 / 0.008, T=2000, alpha=0.25, H_base=4: 250 x 4, 56 x 9, then 496
    H, st = oracle.schedule(oracle.lr_step(2000, 0, 0.8, [1000, 1500], 10.0), 0, 4, 0.25)
    assert list(H) == [4] * 250 + [9] * 56 + [496]
    assert st[249] == 1000 and st[305] == 1504 and st[306] == 2000
    # flat60m: cosine 1e-3 -> 0, T=5000, alpha=0.0175, H_base=4
    H, st = oracle.schedule(oracle.lr_cosine(5000, 0, 1e-3), 0, 4, 0.0175)
    assert list(H) == [306, 311, 330, 366, 434, 578, 994, 1681]
    assert list(st) == [306, 617, 947, 1313, 1747, 2325, 3319, 5000]
    # resmlp: 5 % warm-up, cosine 8e-4 -> 0, T=2000
    H, st = oracle.schedule(oracle.lr_cosine(2000, 100, 8e-4), 100, 4, 0.0175)
    assert list(H) == [478, 583, 939]
    # flat350m: cosine 6e-4 -> 0, T=2000, alpha=0.01, H_base=2
    H, st = oracle.schedule(oracle.lr_cosine(2000, 0, 6e-4), 0, 2, 0.01)
    assert list(H) == [277, 305, 428, 990]


def test_constant_H_when_alpha_is_zero():
    H, st = oracle.schedule(oracle.lr_cosine(103, 0, 0.1), 0, 4, 0.0)
    assert list(H) == [4] * 25 + [3]


def test_schedule_brute_force_random():
    """Eq. (2) re-evaluated with exact rational arithmetic on random tables."""
    from fractions import Fraction
    rng = np.random.default_rng(5)
    for _ in range(50):
        T = int(rng.integers(5, 200))
        Tw = int(rng.integers(0, T // 2 + 1))
        eta = np.sort(rng.uniform(1e-3, 1.0, T))[::-1].copy()
        eta[:Tw] = np.linspace(0, eta[Tw] if Tw < T else 1, Tw, endpoint=False)
        alpha = float(rng.uniform(0.01, 0.5))
        Hb = int(rng.integers(1, 6))
        H, st = oracle.schedule(eta, Tw, Hb, alpha)
        t = 0
        for Hs in H:
            e = eta[max(t, Tw)]
            q = Fraction(alpha) / Fraction(float(e))
            v = q * q
            want = max(Hb, math.floor(v))
            want = min(want, T - t)
            # the floating-point evaluation may differ from the exact one only on a knife edge
            if abs(float(v) - round(float(v))) > 1e-9:
                assert Hs == want
            t += Hs
        assert t == T
