"""Pins for the oracle's readout (CPU only): two-way confidence verdicts, k*, L*, t*."""
import itertools
import math
from decimal import Decimal, getcontext
from pathlib import Path

import numpy as np

from oracle import pv_oracle as orc

GOLDEN = Path(__file__).parent / "golden" / "judge_thresholds.txt"


def paper_taus():
    return [float(x) for x in GOLDEN.read_text().split("\n") if x and not x.startswith("#")]


def p2w_decimal(lc, li):
    """exp(l_C) / (exp(l_C) + exp(l_I)) with 60 digits ("Notation and judge calibration")."""
    getcontext().prec = 60
    ec, ei = Decimal(lc).exp(), Decimal(li).exp()
    return ec / (ec + ei)


def literal_k_star(ok):
    """Largest k such that v_k is Correct and no Incorrect appears earlier (else -1)."""
    best = -1
    for k in range(len(ok)):
        if ok[k] and all(ok[:k]):
            best = k
    return best


def literal_t_star(ok, bounds):
    good = [bounds[k] for k in range(len(ok)) if ok[k]]
    return max(good) if good else 0


def test_margin_rule_equals_p2w_rule():
    rng = np.random.default_rng(5)
    for tau in paper_taus():
        thr = orc.margin_threshold(tau)
        lg = rng.normal(0, 4, size=(400, 2)).astype(np.float32)
        ok = orc.verdicts(lg, thr)
        for (lc, li), o in zip(lg, ok):
            lc, li = float(lc), float(li)
            conf = p2w_decimal(lc, li)
            if abs(conf - Decimal(tau)) < Decimal("1e-12"):
                continue                                    # on the knife edge: skip
            expect = (lc >= li) and (conf >= Decimal(tau))
            assert bool(o) == expect, (tau, lc, li)


def test_threshold_values():
    # tau = 0.5 is the raw argmax rule; the others are monotone and satisfy sigmoid(thr) = tau
    taus = paper_taus()
    assert taus[0] == 0.5 and orc.margin_threshold(0.5) == 0.0
    thr = [orc.margin_threshold(t) for t in taus]
    assert all(a < b for a, b in zip(thr, thr[1:]))
    for t, m in zip(taus, thr):
        assert abs(1.0 / (1.0 + math.exp(-m)) - t) < 1e-15
    assert abs(orc.margin_threshold(0.9) - math.log(9.0)) < 1e-15     # odds 9:1
    assert abs(orc.margin_threshold(0.95) - math.log(19.0)) < 1e-14   # odds 19:1


def test_tie_counts_as_correct_and_config1_rule():
    # tie l_C = l_I with tau = 0.5 -> Correct;  "reject if logit < 0" with l_I = 0
    lg = np.array([[0.0, 0.0], [-1e-30, 0.0], [1e-30, 0.0], [2.5, 2.5]], dtype=np.float32)
    assert list(orc.verdicts(lg, 0.0)) == [True, False, True, True]
    # a negative threshold (tau < 0.5) can never turn a raw Incorrect into Correct
    assert list(orc.verdicts(np.array([[0.0, 0.5]], dtype=np.float32), -2.0)) == [False]


def test_exhaustive_patterns():
    for K in range(0, 11):
        bounds = [3 * k + 2 for k in range(K)]
        for pattern in itertools.product([True, False], repeat=K):
            lg = np.array([[4.0, 0.0] if c else [0.0, 1.0] for c in pattern], dtype=np.float32).reshape(K, 2)
            r0 = orc.first_reject(lg, [K], [bounds], 1.0, mode=0)[0]
            r1 = orc.first_reject(lg, [K], [bounds], 1.0, mode=1)[0]
            ks = literal_k_star(list(pattern))
            assert r0[1] == ks
            assert r0[0] == ks + 1
            assert r0[2] == (bounds[ks] if ks >= 0 else 0)
            assert r0[3] == sum(1 for c in pattern if not c)
            assert r1[2] == literal_t_star(list(pattern), bounds)
            assert r1[0] == r0[0] and r1[3] == r0[3]


def test_hand_patterns_and_batching():
    C, I = [5.0, 0.0], [0.0, 5.0]
    lg = np.array([C, C, I, C,      # request 0: (C,C,I,C)
                   C, C, C,         # request 1: all Correct
                   I, C],           # request 2: first is Incorrect
                  dtype=np.float32)
    bounds = [[10, 20, 30, 40], [5, 6, 7], [8, 9]]
    r = orc.first_reject(lg, [4, 3, 2], bounds, 2.0, mode=0)
    assert r.dtype == np.int32 and r.shape == (3, 4)
    assert list(r[0]) == [2, 1, 20, 1]
    assert list(r[1]) == [3, 2, 7, 0]          # first_reject = K when nothing is rejected
    assert list(r[2]) == [0, -1, 0, 1]         # k* = -1, L* = 0: restart
    r = orc.first_reject(lg, [4, 3, 2], bounds, 2.0, mode=1)
    assert list(r[0]) == [2, 3, 40, 1]         # main-text rule picks the later Correct prefix
    assert list(r[2]) == [0, 1, 9, 1]
    # the threshold downgrades a weak Correct
    weak = np.array([[1.0, 0.0], [5.0, 0.0]], dtype=np.float32)
    assert list(orc.first_reject(weak, [2], [[3, 4]], 2.0, 0)[0]) == [0, -1, 0, 1]
    assert list(orc.first_reject(weak, [2], [[3, 4]], 0.5, 0)[0]) == [2, 1, 4, 0]
    # K = 0
    assert list(orc.first_reject(np.zeros((0, 2), np.float32), [0], [[]], 0.0, 0)[0]) == [0, -1, 0, 0]


def test_uniform_boundaries_match_adopted_length_formula():
    # L* = min(T, Delta * floor(max(0, k* + 1 - eta))) with eta = 0 and boundaries every Delta
    T, Delta = 130, 40
    K = math.ceil(T / Delta)
    bounds = [min(T, Delta * (k + 1)) for k in range(K)]
    for first_bad in range(K + 1):
        lg = np.array([[9.0, 0.0] if k < first_bad else [0.0, 9.0] for k in range(K)], dtype=np.float32)
        k_star = first_bad - 1
        L = min(T, Delta * math.floor(max(0, k_star + 1 - 0.0)))
        assert orc.first_reject(lg, [K], [bounds], 1.0, 0)[0][2] == L
