"""Pins for the oracle's decision policy (CPU only): the rho / kappa reject rules, the adopted-prefix
formula with rollback, the stage decisions of the detailed algorithm, and the judge logits.

Nothing here re-calls the oracle's own formulas: the rules are transcribed literally from the text
(fractions with exact rationals, runs by scanning, stages as nested ifs on probabilities computed
with 60-digit decimals), and the closed form of the adopted-prefix equation is evaluated for uniform
chunking."""
import itertools
import math
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np

from oracle import pv_oracle as orc

C_, I_ = [9.0, 0.0], [0.0, 9.0]


def p2w(lc, li):
    getcontext().prec = 60
    ec, ei = Decimal(float(lc)).exp(), Decimal(float(li)).exp()
    return ec / (ec + ei)


def literal_rules(pattern, rho, kappa):
    """Fraction of Incorrect chunks exceeds rho, or the trailing run of Incorrect chunks reaches kappa."""
    K = len(pattern)
    n_inc = sum(1 for c in pattern if not c)
    run = 0
    while run < K and not pattern[K - 1 - run]:
        run += 1
    frac = K > 0 and Fraction(n_inc, K) > Fraction(str(rho))     # rho as the decimal number written
    return (frac or (kappa > 0 and run >= kappa)), n_inc, run


def test_chunk_run_rules_exhaustive():
    for K in range(0, 11):
        for pattern in itertools.product([True, False], repeat=K):
            for rho in (0.0, 0.2, 0.25, 0.3, 0.5, 1.0):
                for kappa in (0, 2, 3):
                    got = orc.chunk_run_rules(np.array(pattern, dtype=bool), rho, kappa)
                    assert got == literal_rules(pattern, rho, kappa), (pattern, rho, kappa)


def test_rule_boundaries():
    # "exceeds rho": exactly rho does not reject; "reaches kappa": exactly kappa does
    ok = np.array([True, True, False, True], dtype=bool)               # 1 of 4 Incorrect
    assert orc.chunk_run_rules(ok, 0.25, 5)[0] is False
    assert orc.chunk_run_rules(ok, 0.2499, 5)[0] is True
    ok = np.array([True, True, True, True, True, True, True, True, False, False], dtype=bool)
    assert orc.chunk_run_rules(ok, 0.3, 2) == (True, 2, 2)             # the paper's rho = 0.30, kappa = 2
    assert orc.chunk_run_rules(ok, 0.3, 3) == (False, 2, 2)


def test_adopted_prefix_closed_form():
    # L* = min(T, Delta * floor(max(0, k* + 1 - eta))) for chunks of Delta tokens
    for T, Delta in ((130, 40), (160, 40), (7, 3), (40, 40)):
        K = math.ceil(T / Delta)
        bounds = [min(T, Delta * (k + 1)) for k in range(K)]
        for k_star in range(-1, K):
            for eta in (0.0, 0.5, 1.0, 1.5, 2.0, 7.0):
                want = min(T, Delta * math.floor(max(0.0, k_star + 1 - eta)))
                assert orc.adopted_prefix(k_star, eta, bounds) == want, (T, Delta, k_star, eta)


def literal_pipeline(chunk_lg, full_lg, bounds, taus, rho, kappa, eta, K_sd):
    """Stages 2-6 of the detailed algorithm written with probabilities, as in the listing."""
    tau_F, tau_F_rx, tau_C_rx, tau_P, tau_sd = taus
    K = len(chunk_lg)
    pF = p2w(*full_lg)
    vF = full_lg[0] >= full_lg[1] and pF >= Decimal(tau_F)
    if vF:
        return orc.LABEL_SM, 2, None
    tau_sd_K = min(tau_sd + 0.02 * (K - 1), tau_F_rx)
    if 1 <= K <= K_sd and pF >= Decimal(tau_sd_K):
        return orc.LABEL_SM, 3, None
    ps = [p2w(*lg) for lg in chunk_lg]
    v = [lg[0] >= lg[1] and p >= Decimal(tau_P) for lg, p in zip(chunk_lg, ps)]
    k_star = -1
    for k in range(K):
        if v[k] and all(v[:k]):
            k_star = k
    p_min = min(ps) if ps else Decimal(1)
    if pF >= Decimal(tau_F_rx) and p_min >= Decimal(tau_C_rx):
        return orc.LABEL_SM, 5, None
    m = math.floor(max(0.0, k_star + 1 - eta))
    L = bounds[m - 1] if m >= 1 else 0
    return (orc.LABEL_SM_LG if L > 0 else orc.LABEL_LG), 6, L


def policy_kwargs(taus, rho, kappa, eta, K_sd, premature=False):
    tau_F, tau_F_rx, tau_C_rx, tau_P, tau_sd = taus
    return dict(margin_chunk=orc.margin_threshold(tau_P), margin_chunk_relaxed=orc.margin_threshold(tau_C_rx),
                margin_full=orc.margin_threshold(tau_F), margin_full_relaxed=orc.margin_threshold(tau_F_rx),
                margin_short=orc.short_draft_margins(tau_sd, tau_F_rx, K_sd), rho=rho, kappa=kappa, eta=eta,
                premature=premature)


QWEN = (0.998, 0.95, 0.90, 0.985, 0.95)      # tau_F, tau_F^rx, tau_C^rx, tau_P, tau_sd (hyper-parameter table)
GLM = (0.95, 0.90, 0.83, 0.88, 0.90)


def test_pipeline_random_against_literal_transcription():
    rng = np.random.default_rng(21)
    for trial in range(3000):
        taus, rho = (QWEN, 0.30) if trial % 2 else (GLM, 0.20)
        K = int(rng.integers(0, 7))
        # margins spread around the thresholds (logit 0.83 .. 0.998 = 1.6 .. 6.2), never within 1e-6 of one
        chunk = np.stack([rng.normal(0, 2, K), rng.normal(0, 2, K)], axis=1).astype(np.float32)
        chunk[:, 0] += rng.choice([0.0, 3.0, 6.0, 9.0], size=K).astype(np.float32)
        full = np.array([[rng.normal(0, 1) + rng.choice([0.0, 3.0, 5.0, 8.0]), rng.normal(0, 1)]], dtype=np.float32)
        bounds = sorted(int(x) for x in rng.integers(0, 200, K))
        eta = float(rng.choice([0.0, 0.0, 1.0, 0.5]))
        want = literal_pipeline([tuple(map(float, r)) for r in chunk], tuple(map(float, full[0])), bounds,
                                taus, rho, 2, eta, 2)
        got = orc.decide(chunk, full, [K], [bounds], **policy_kwargs(taus, rho, 2, eta, 2))[0]
        assert (got[0], got[1]) == want[:2], (trial, got, want)
        if want[2] is not None:
            assert got[2] == want[2]
        assert got[11] == K


def test_pipeline_hand_cases():
    kw = policy_kwargs(QWEN, 0.30, 2, 0.0, 2)
    chunk = np.array([C_, C_, I_, C_], dtype=np.float32)
    bounds = [[40, 80, 120, 150]]
    strong, weak, mid = [[9.0, 0.0]], [[0.0, 1.0]], [[3.5, 0.0]]       # p = 0.9999, 0.27, 0.97
    assert list(orc.decide(chunk, np.array(strong, np.float32), [4], bounds, **kw)[0][:3]) == [orc.LABEL_SM, 2, 80]
    r = orc.decide(chunk, np.array(weak, np.float32), [4], bounds, **kw)[0]
    assert list(r) == [orc.LABEL_SM_LG, 6, 80, 1, 2, 1, 0, 0, 1, 0, 2, 4]
    # relaxed accept needs every chunk above tau_C^rx
    allc = np.array([C_, C_, C_], dtype=np.float32)
    assert list(orc.decide(allc, np.array(mid, np.float32), [3], [[40, 80, 100]], **kw)[0][:2]) == [orc.LABEL_SM, 5]
    onebad = np.array([C_, [2.0, 0.0], C_], dtype=np.float32)            # p = 0.88 < 0.90
    r = orc.decide(onebad, np.array(mid, np.float32), [3], [[40, 80, 100]], **kw)[0]
    assert list(r[:5]) == [orc.LABEL_SM_LG, 6, 40, 0, 1] and r[8] == 1 and r[10] == 1
    # short draft: K <= 2 and p_F >= min(tau_sd + 0.02 (K - 1), tau_F^rx) = 0.95
    short = np.array([I_, I_], dtype=np.float32)
    assert list(orc.decide(short, np.array(mid, np.float32), [2], [[40, 70]], **kw)[0][:2]) == [orc.LABEL_SM, 3]
    assert list(orc.decide(short, np.array([[2.5, 0.0]], np.float32), [2], [[40, 70]], **kw)[0][:3]) == \
        [orc.LABEL_LG, 6, 0]                                             # p_F = 0.924: restart from the prompt
    # rollback by one chunk
    kw1 = policy_kwargs(QWEN, 0.30, 2, 1.0, 2)
    assert orc.decide(chunk, np.array(weak, np.float32), [4], bounds, **kw1)[0][2] == 40


def test_premature_exit():
    kw = policy_kwargs(QWEN, 0.20, 2, 0.0, 2, premature=True)           # rho_p = 0.20
    go = np.array([C_] * 8, dtype=np.float32)
    assert list(orc.decide(go, None, [8], [list(range(40, 321, 40))], **kw)[0][:2]) == [-1, 0]
    two_bad_tail = np.array([C_] * 6 + [I_, I_], dtype=np.float32)       # trailing run reaches kappa
    r = orc.decide(two_bad_tail, None, [8], [list(range(40, 321, 40))], **kw)[0]
    assert list(r[:4]) == [orc.LABEL_SM_LG, 1, 240, 5] and r[7] == 1 and r[9] == -1
    # three chunks below the relaxed chunk threshold abort even when the strict rules pass
    soft = [2.0, 0.0]                                                    # p = 0.88: Incorrect at 0.985, below 0.90
    kw_loose = dict(kw, margin_chunk=orc.margin_threshold(0.5), rho=0.9, kappa=0)
    three_soft = np.array([C_, soft, C_, soft, C_, soft, C_, C_], dtype=np.float32)
    r = orc.decide(three_soft, None, [8], [list(range(40, 321, 40))], **kw_loose)[0]
    assert r[7] == 0 and r[8] == 3 and r[1] == 1
    two_soft = np.array([C_, soft, C_, soft, C_, C_, C_, C_], dtype=np.float32)
    assert orc.decide(two_soft, None, [8], [list(range(40, 321, 40))], **kw_loose)[0][1] == 0


def test_short_draft_margins():
    m = orc.short_draft_margins(0.90, 0.95, 4)
    for K, got in enumerate(m, start=1):
        tau = min(0.90 + 0.02 * (K - 1), 0.95)
        assert got == math.log(tau / (1 - tau))
    assert m[3] == orc.margin_threshold(0.95)                            # capped by the relaxed full threshold


def test_judge_logits_against_exact_rational_dot():
    rng = np.random.default_rng(3)
    hidden = rng.integers(-8, 9, size=(10, 24)).astype(np.float64) / 4
    w2 = rng.integers(-8, 9, size=(2, 24)).astype(np.float64) / 8
    rows = [9, 0, 3]
    got = orc.judge_logits(hidden, w2, np.array(rows))
    for i, r in enumerate(rows):
        for c in range(2):
            want = sum(Fraction(hidden[r, j]) * Fraction(w2[c, j]) for j in range(24))
            assert Fraction(got[i, c]) == want                           # dyadic inputs: exact in fp64


# --- thresholds exactly at equality, and the tie rule of the least confident chunk.  Logits are dyadic,
# so every margin l_C - l_I is exact in fp64 and can be made to coincide with a threshold to the bit.
# What happens at equality is written out below from the listing's comparisons, not from the oracle.

def _edge_kwargs(**over):
    kw = dict(margin_chunk=2.25, margin_chunk_relaxed=1.5, margin_full=6.0, margin_full_relaxed=3.0,
              margin_short=[3.5, 3.75], rho=0.9, kappa=0, eta=0.0)
    kw.update(over)
    return kw


def _lg(*margins):
    """Logit pairs (1 + m, 1) with the given dyadic margins."""
    return np.array([[1.0 + m, 1.0] for m in margins], dtype=np.float32).reshape(-1, 2)


def test_chunk_threshold_at_equality_accepts():
    # Stage 4 verdict: v_k Correct iff l_C >= l_I and p_2w >= tau_P.  A chunk whose confidence EQUALS
    # tau_P is Correct; one ulp below is Incorrect.
    below = float(np.nextafter(np.float32(3.25), np.float32(0)) - np.float32(1.0))   # margin just under 2.25
    bounds = [[10, 20, 30]]
    full = _lg(0.0)                                     # weak full verdict: falls through to Stage 6
    at = orc.decide(_lg(2.25, 2.25, 2.25), full, [3], bounds, **_edge_kwargs())[0]
    assert list(at[3:6]) == [2, 3, 0]                   # k* = 2, first_reject = K, no Incorrect chunk
    assert list(at[:3]) == [orc.LABEL_SM_LG, 6, 30]
    chunk = _lg(2.25, 2.25, 2.25)
    chunk[1, 0] = np.nextafter(np.float32(3.25), np.float32(0))
    assert float(chunk[1, 0]) - 1.0 == below < 2.25
    un = orc.decide(chunk, full, [3], bounds, **_edge_kwargs())[0]
    assert list(un[3:6]) == [0, 1, 1] and un[2] == 10   # chunk 1 Incorrect: k* = 0, L* = p_0
    # the plain readout takes the same decision at equality
    assert list(orc.first_reject(_lg(2.25, 2.25), [2], [[10, 20]], 2.25, 0)[0]) == [2, 1, 20, 0]


def test_relaxed_chunk_threshold_is_strict_below():
    # premature exit counts chunks with p_2w < tau_C^rx: a chunk AT the relaxed threshold is not
    # counted; Stage 5 needs p_min >= tau_C^rx, which the same chunk satisfies.
    kw = _edge_kwargs(margin_chunk=0.0, premature=True)
    three_at = _lg(1.5, 1.5, 1.5, 4.0)
    r = orc.decide(three_at, None, [4], [[5, 10, 15, 20]], **kw)[0]
    assert r[8] == 0 and list(r[:2]) == [-1, 0]          # nothing below: keep drafting
    three_under = _lg(1.25, 1.25, 1.25, 4.0)
    r = orc.decide(three_under, None, [4], [[5, 10, 15, 20]], **kw)[0]
    assert r[8] == 3 and r[1] == 1                       # three below: abort
    # Stage 5 with p_F at tau_F^rx and p_min at tau_C^rx, both exactly: relaxed accept
    kw5 = _edge_kwargs(margin_chunk=0.0)
    r = orc.decide(_lg(1.5, 4.0, 4.0), _lg(3.0), [3], [[5, 10, 15]], **kw5)[0]
    assert list(r[:2]) == [orc.LABEL_SM, 5] and r[8] == 0
    r = orc.decide(_lg(1.25, 4.0, 4.0), _lg(3.0), [3], [[5, 10, 15]], **kw5)[0]
    assert list(r[:2]) == [orc.LABEL_SM_LG, 6] and r[8] == 1


def test_full_thresholds_at_equality():
    chunk = _lg(4.0, -1.0, 4.0, 4.0)                     # K = 4 > K^sd = 2; chunk 1 Incorrect and below relaxed
    bounds = [[5, 10, 15, 20]]
    # Stage 2: p_F >= tau_F accepts at equality
    assert list(orc.decide(chunk, _lg(6.0), [4], bounds, **_edge_kwargs())[0][:2]) == [orc.LABEL_SM, 2]
    assert orc.decide(chunk, _lg(6.0), [4], bounds, **_edge_kwargs())[0][9] == 1
    r = orc.decide(chunk, _lg(5.75), [4], bounds, **_edge_kwargs())[0]
    assert list(r[:3]) == [orc.LABEL_SM_LG, 6, 5] and r[9] == 0
    # Stage 5: p_F >= tau_F^rx at equality (every chunk above the relaxed chunk threshold)
    good = _lg(4.0, 4.0, 4.0, 4.0)
    assert list(orc.decide(good, _lg(3.0), [4], bounds, **_edge_kwargs())[0][:2]) == [orc.LABEL_SM, 5]
    assert list(orc.decide(good, _lg(2.75), [4], bounds, **_edge_kwargs())[0][:3]) == [orc.LABEL_SM_LG, 6, 20]
    # Stage 3: K <= K^sd and p_F >= tau_sd^(K) at equality, per chunk count
    bad2, bad1 = _lg(-1.0, -1.0), _lg(-1.0)
    assert list(orc.decide(bad2, _lg(3.75), [2], [[5, 9]], **_edge_kwargs())[0][:2]) == [orc.LABEL_SM, 3]
    assert list(orc.decide(bad2, _lg(3.5), [2], [[5, 9]], **_edge_kwargs())[0][:3]) == [orc.LABEL_LG, 6, 0]
    assert list(orc.decide(bad1, _lg(3.5), [1], [[5]], **_edge_kwargs())[0][:2]) == [orc.LABEL_SM, 3]
    assert list(orc.decide(bad1, _lg(3.25), [1], [[5]], **_edge_kwargs())[0][:3]) == [orc.LABEL_LG, 6, 0]
    # K = K^sd + 1 never takes Stage 3
    assert orc.decide(_lg(-1.0, -1.0, -1.0), _lg(3.75), [3], [[5, 9, 12]], **_edge_kwargs())[0][1] == 6


def test_least_confident_chunk_first_of_equals():
    # output [10]: index of the least confident chunk; of several equal minima the first
    r = orc.decide(_lg(4.0, 0.5, 3.0, 0.5, 0.5), _lg(0.0), [5], [[1, 2, 3, 4, 5]], **_edge_kwargs())[0]
    assert r[10] == 1
    r = orc.decide(_lg(0.5, 0.5), _lg(0.0), [2], [[1, 2]], **_edge_kwargs())[0]
    assert r[10] == 0
    r = orc.decide(_lg(4.0, 3.0, -2.0), _lg(0.0), [3], [[1, 2, 3]], **_edge_kwargs())[0]
    assert r[10] == 2
    assert orc.decide(_lg(), _lg(0.0), [0], [[]], **_edge_kwargs())[0][10] == -1


def test_short_draft_thresholds_are_the_listed_taus():
    # tau_sd^(K) = min(tau_sd + 0.02 (K - 1), tau_F^rx): with tau_sd = 0.90 and tau_F^rx = 0.95 the
    # thresholds for K = 1..4 are 0.90, 0.92, 0.94, 0.95 (typed here, not computed); the margin of
    # each must have exactly that two-way confidence (60-digit logistic function).
    getcontext().prec = 60
    for m, tau in zip(orc.short_draft_margins(0.90, 0.95, 4), ("0.90", "0.92", "0.94", "0.95")):
        conf = 1 / (1 + (-Decimal(m)).exp())
        assert abs(conf - Decimal(tau)) < Decimal("1e-15"), (m, tau)
    for m, tau in zip(orc.short_draft_margins(0.95, 0.95, 2), ("0.95", "0.95")):
        assert abs(1 / (1 + (-Decimal(m)).exp()) - Decimal(tau)) < Decimal("1e-15")
