"""GPU parity of pv_judge_logits (floating point, tolerance below) and pv_decide (bit-exact) against
the oracle, through the C ABI."""
import itertools

import numpy as np
import pytest
import torch

import pv_workloads as wl
from oracle import pv_oracle as orc
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")

QWEN = (0.998, 0.95, 0.90, 0.985, 0.95)      # tau_F, tau_F^rx, tau_C^rx, tau_P, tau_sd
GLM = (0.95, 0.90, 0.83, 0.88, 0.90)


def policies(taus, rho, kappa, eta, K_sd, premature=False):
    tau_F, tau_F_rx, tau_C_rx, tau_P, tau_sd = taus
    kw = dict(margin_chunk=orc.margin_threshold(tau_P), margin_chunk_relaxed=orc.margin_threshold(tau_C_rx),
              margin_full=orc.margin_threshold(tau_F), margin_full_relaxed=orc.margin_threshold(tau_F_rx),
              margin_short=orc.short_draft_margins(tau_sd, tau_F_rx, K_sd), rho=rho, kappa=kappa, eta=eta,
              premature=premature)
    return kw, pv.make_policy(kw["margin_chunk"], kw["margin_chunk_relaxed"], kw["margin_full"],
                              kw["margin_full_relaxed"], kw["margin_short"], rho, kappa, eta, 3, premature)


def verifier_for(pr):
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.float32, seed=1)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    return ver


def check_decide(pr, chunk, full):
    ver = verifier_for(pr)
    lg = torch.from_numpy(chunk).to(ver.device)
    fl = torch.from_numpy(full).to(ver.device)
    for taus, rho in ((QWEN, 0.30), (GLM, 0.20)):
        for eta in (0.0, 1.0, 0.5):
            for kappa, K_sd in ((2, 2), (0, 0), (3, 8)):
                kw, pol = policies(taus, rho, kappa, eta, K_sd)
                got = ver.decide(lg, fl, pol).cpu().numpy()
                exp = orc.decide(chunk, full, pr.num_segments, pr.boundaries, **kw)
                assert np.array_equal(got, exp), (taus, eta, kappa, K_sd)
                kw, pol = policies(taus, rho, kappa, eta, K_sd, premature=True)
                got = ver.decide(lg, None, pol).cpu().numpy()
                exp = orc.decide(chunk, None, pr.num_segments, pr.boundaries, **kw)
                assert np.array_equal(got, exp), ("premature", taus, eta, kappa)


def test_decide_all_verdict_patterns():
    # every Correct / soft / Incorrect pattern of 5 chunks as one batch of 243 requests
    levels = ([9.0, 0.0], [2.0, 0.0], [0.0, 9.0])
    pats = list(itertools.product(range(3), repeat=5))
    B = len(pats)
    pr = wl.Problem([8] * B, [200] * B, [5] * B, [4] * B, [[40, 80, 120, 160, 200]] * B)
    chunk = np.array([levels[c] for p in pats for c in p], dtype=np.float32)
    rng = np.random.default_rng(4)
    full = np.stack([rng.choice([0.0, 2.5, 3.5, 9.0], size=B), np.zeros(B)], axis=1).astype(np.float32)
    check_decide(pr, chunk, full)


def test_decide_ragged_random_and_named():
    rng = np.random.default_rng(8)
    B = 40
    K = [int(x) for x in rng.integers(0, 12, B)]
    T = [int(x) for x in rng.integers(1, 400, B)]
    bounds = [sorted(int(x) for x in rng.integers(0, T[b] + 1, K[b])) for b in range(B)]
    pr = wl.Problem([3] * B, T, K, [2] * B, bounds)
    n = sum(K)
    chunk = np.stack([rng.normal(3, 4, n), rng.normal(0, 1, n)], axis=1).astype(np.float32)
    full = np.stack([rng.normal(3, 3, B), rng.normal(0, 1, B)], axis=1).astype(np.float32)
    check_decide(pr, chunk, full)
    for name in ("tiny", "8b", "ragged", "14b", "70b"):
        w = wl.make(name)
        prn = w.problem
        full = np.stack([rng.normal(3, 3, prn.batch), rng.normal(0, 1, prn.batch)], axis=1).astype(np.float32)
        check_decide(prn, w.logits.numpy(), full)


def test_decide_thresholds_at_exact_equality():
    # dyadic logits: the fp64 margin l_C - l_I coincides with a threshold to the bit.  At equality a
    # chunk is Correct (>= tau_P), is not counted as below the relaxed chunk threshold (< tau_C^rx), and
    # the full-answer confidence passes the strict, short-draft and relaxed gates (>=); one float below,
    # none of that holds.  Expected values from the oracle, whose equality cases are pinned on the CPU.
    def lg(*margins):
        return np.array([[1.0 + m, 1.0] for m in margins], dtype=np.float32).reshape(-1, 2)
    under = float(np.nextafter(np.float32(3.25), np.float32(0))) - 1.0          # just below 2.25
    cases = [  # (chunk margins, full margin)
        ((2.25, 2.25, 2.25), 0.0), ((2.25, under, 2.25), 0.0), ((1.5, 1.5, 1.5, 4.0), 0.0),
        ((1.25, 1.25, 1.25, 4.0), 0.0), ((1.5, 4.0, 4.0), 3.0), ((1.25, 4.0, 4.0), 3.0),
        ((4.0, -1.0, 4.0, 4.0), 6.0), ((4.0, -1.0, 4.0, 4.0), 5.75), ((4.0, 4.0, 4.0, 4.0), 3.0),
        ((4.0, 4.0, 4.0, 4.0), 2.75), ((-1.0, -1.0), 3.75), ((-1.0, -1.0), 3.5), ((-1.0,), 3.5), ((-1.0,), 3.25),
        ((4.0, 0.5, 3.0, 0.5, 0.5), 0.0), ((0.5, 0.5), 0.0), ((), 0.0),
    ]
    K = [len(c[0]) for c in cases]
    pr = wl.Problem([2] * len(cases), [40] * len(cases), K, [1] * len(cases),
                    [[5 * (k + 1) for k in range(n)] for n in K])
    chunk = np.concatenate([lg(*c[0]) for c in cases])
    chunk[4, 0] = np.nextafter(np.float32(3.25), np.float32(0))                 # the `under` entry, exactly
    full = np.concatenate([lg(c[1]) for c in cases])
    ver = verifier_for(pr)
    for premature in (False, True):
        for margin_chunk in (2.25, 0.0):
            kw = dict(margin_chunk=margin_chunk, margin_chunk_relaxed=1.5, margin_full=6.0, margin_full_relaxed=3.0,
                      margin_short=[3.5, 3.75], rho=0.9, kappa=0, eta=0.0, premature=premature)
            pol = pv.make_policy(margin_chunk, 1.5, 6.0, 3.0, [3.5, 3.75], 0.9, 0, 0.0, 3, premature)
            got = ver.decide(torch.from_numpy(chunk).to(ver.device),
                             None if premature else torch.from_numpy(full).to(ver.device), pol).cpu().numpy()
            exp = orc.decide(chunk, None if premature else full, pr.num_segments, pr.boundaries, **kw)
            assert np.array_equal(got, exp), (premature, margin_chunk, got, exp)
    # and the plain readout at the same equality
    got = ver.first_reject(torch.from_numpy(chunk).to(ver.device), 2.25, 0).cpu().numpy()
    assert np.array_equal(got, orc.first_reject(chunk, pr.num_segments, pr.boundaries, 2.25, 0))
    assert got[0].tolist() == [3, 2, 15, 0] and got[1].tolist() == [1, 0, 5, 1]


def test_decide_agrees_with_first_reject():
    w = wl.make("ragged")
    pr = w.problem
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    lg = w.logits.to(ver.device)
    kw, pol = policies(QWEN, 0.3, 2, 0.0, 2, premature=True)
    d = ver.decide(lg, None, pol).cpu().numpy()
    r = ver.first_reject(lg, kw["margin_chunk"], 0).cpu().numpy()
    assert np.array_equal(d[:, [4, 3, 2, 5]], r)                 # first_reject, k*, L* (eta = 0), n_incorrect


@pytest.mark.parametrize("hidden_size", [64, 4096, 5120, 8200])
def test_judge_logits(hidden_size):
    # tolerance: fp32 accumulation of exact bf16 products, 64 partial sums of hidden_size/64 terms and a
    # 6-level tree: |err| <= (hidden_size/64 + 6) * 2^-24 * sum |h_i w_i|, far below the 1e-5 * sum used
    rng = np.random.default_rng(hidden_size)
    pr = wl.Problem([5, 0, 17], [40, 9, 64], [4, 0, 7], [5, 1, 3], [[1, 20, 40, 40], [], [0, 3, 9, 30, 31, 60, 64]])
    ver = verifier_for(pr)
    hidden = torch.from_numpy(rng.normal(0, 1, (pr.total_tokens, hidden_size)).astype(np.float32)).bfloat16()
    w2 = torch.from_numpy(rng.normal(0, 0.05, (2, hidden_size)).astype(np.float32)).bfloat16()
    got = ver.judge_logits(hidden.to(ver.device), w2.to(ver.device)).cpu().numpy().astype(np.float64)
    _, rows = gc.oracle_plan_arrays(pr)
    h64, w64 = hidden.double().numpy(), w2.double().numpy()
    exp = orc.judge_logits(h64, w64, rows)
    bound = 1e-5 * (np.abs(h64[rows])[:, None, :] * np.abs(w64)[None, :, :]).sum(axis=2) + 1e-30
    assert got.shape == exp.shape == (pr.total_segments, 2)
    assert (np.abs(got - exp) <= bound).all(), np.abs(got - exp).max()
    # and the logits feed the readout unchanged
    again = ver.judge_logits(hidden.to(ver.device), w2.to(ver.device)).cpu().numpy()
    assert np.array_equal(again.astype(np.float64), got)         # bit-reproducible
