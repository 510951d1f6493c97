"""Pins for the oracle's interleaved packing (CPU only): prefix | (C_k | End_k)_k of appendix
"Parallel partial verify".

None of them reuses the oracle's own construction: a literal pairwise predicate over token
identities on exhaustive tiny inputs, closed-form counts, the stand-alone equivalence (an End
slot's rows equal a library causal attention over [prefix, C_1..C_k, End_k] alone), and the fact
that the interleaved packing is a reordering of the appended one (same tokens, same visibility,
same positions), checked with a permutation built here from the token identities.
"""
import itertools
import math

import numpy as np
import torch

from oracle import pv_oracle as orc
import pv_workloads as wl
from tests.test_oracle_attention import library_causal, library_causal_lse, rope_complex


def packed_identities(P, T, S, bounds):
    """Token identities of the interleaved packing, rebuilt here by insertion: start from the
    plain sequence prefix + draft and insert copy k of the suffix after draft token p_k - 1
    (after the prefix if p_k = 0), later copies behind earlier ones."""
    seq = [("prefix", i) for i in range(P)] + [("draft", t) for t in range(T)]
    for k in reversed(range(len(bounds))):
        at = P + bounds[k]
        seq[at:at] = [("suffix", k, a) for a in range(S)]
    return seq


def literal_visible(qi, kj, i, j, bounds):
    """The appendix's sentence for End slots plus ordinary causality for everything else."""
    if j > i:
        return False
    if kj[0] == "prefix":
        return True
    if qi[0] == "suffix":
        k = qi[1]
        if kj[0] == "draft":
            return kj[1] < bounds[k]                  # own prefix C_1..C_k = first p_k draft tokens
        return kj[1] == k                             # only its own copy
    return kj[0] == "draft"                           # prefix/draft rows never see a suffix copy


def all_boundary_lists(T, K):
    return itertools.combinations_with_replacement(range(T + 1), K)


def test_insertion_order_matches_and_mask_is_literal_on_tiny_inputs():
    n = 0
    for P, T, S in itertools.product([0, 1, 2], [1, 2, 4, 5], [1, 2, 3]):
        for K in range(0, 4):
            for bounds in all_boundary_lists(T, K):
                ids = packed_identities(P, T, S, list(bounds))
                toks = orc.interleaved_tokens(P, T, S, list(bounds))
                assert len(ids) == len(toks) == P + T + K * S
                for a, b in zip(ids, toks):
                    assert (a[0], b[0]) in (("prefix", "q"), ("draft", "c"), ("suffix", "e"))
                    assert a[-1] == b[-1] and (a[0] != "suffix" or a[1] == b[1])
                M = orc.dense_mask_interleaved(P, T, S, list(bounds))
                N = len(ids)
                ref = np.array([[literal_visible(ids[i], ids[j], i, j, bounds) for j in range(N)]
                                for i in range(N)], dtype=np.uint8)
                assert np.array_equal(M, ref), (P, T, S, bounds)
                n += 1
    assert n > 1000


def to_appended(P, T, S, bounds):
    """perm[i_appended] = index of the same token in the interleaved packing."""
    ids = packed_identities(P, T, S, bounds)
    where = {t: i for i, t in enumerate(ids)}
    order = [("prefix", i) for i in range(P)] + [("draft", t) for t in range(T)] + \
            [("suffix", k, a) for k in range(len(bounds)) for a in range(S)]
    return np.array([where[t] for t in order])


def test_interleaved_is_a_reordering_of_the_appended_packing():
    rng = np.random.default_rng(5)
    for _ in range(40):
        P, T, S, K = int(rng.integers(0, 9)), int(rng.integers(1, 40)), int(rng.integers(1, 7)), int(rng.integers(0, 7))
        bounds = sorted(int(x) for x in rng.integers(0, T + 1, K))
        perm = to_appended(P, T, S, bounds)
        MA = orc.dense_mask(P, T, S, bounds)
        MB = orc.dense_mask_interleaved(P, T, S, bounds)
        assert np.array_equal(MB[np.ix_(perm, perm)], MA)
        assert np.array_equal(orc.positions_interleaved(P, T, S, bounds)[perm], orc.positions(P, T, S, bounds))
        assert np.array_equal(orc.judge_rows_interleaved(P, T, S, bounds), perm[orc.judge_rows(P, T, S, K)])


def test_counts_and_judge_rows_closed_form():
    P, T, S, bounds = 7, 50, 4, [0, 9, 9, 30, 50]
    M = orc.dense_mask_interleaved(P, T, S, bounds)
    c = P + T
    assert int(M.sum()) == c * (c + 1) // 2 + sum(S * (P + p) + S * (S + 1) // 2 for p in bounds)
    jr = orc.judge_rows_interleaved(P, T, S, bounds)
    # copy k sits behind the prefix, p_k draft tokens and k earlier copies
    assert list(jr) == [P + p + k * S + S - 1 for k, p in enumerate(bounds)]
    for k, p in enumerate(bounds):
        for a in range(S):
            assert int(M[P + p + k * S + a].sum()) == P + p + a + 1
    pos = orc.positions_interleaved(P, T, S, bounds)
    assert [int(pos[r]) for r in jr] == [P + p + S - 1 for p in bounds]
    # no boundaries: the plain causal sequence
    assert np.array_equal(orc.dense_mask_interleaved(3, 9, 2, []), np.tril(np.ones((12, 12), dtype=np.uint8)))
    assert np.array_equal(orc.positions_interleaved(3, 9, 2, []), np.arange(12))


def standalone_check(w, atol=1e-11):
    """Every End slot equals a stand-alone causal pass over [prefix, draft[:p_k], its copy]; prefix
    and draft rows equal a causal pass over prefix + draft alone."""
    pr = w.problem
    G = w.n_q_heads // w.n_kv_heads
    scale = 1.0 / math.sqrt(w.head_dim)
    q = w.q.double().numpy(); k = w.k.double().numpy(); v = w.v.double().numpy()
    O, LSE = orc.masked_attention(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len, pr.boundaries,
                                  q, k, v, rope_theta=w.rope_theta, layout=orc.LAYOUT_INTERLEAVED,
                                  return_lse=True)
    cu = pr.token_offsets()
    worst = 0.0
    for b in range(pr.batch):
        P, T, K, S = pr.prompt_len[b], pr.draft_len[b], pr.num_segments[b], pr.segment_len[b]
        bounds = pr.boundaries[b]
        ids = packed_identities(P, T, S, bounds)
        where = {t: i for i, t in enumerate(ids)}
        qb, kb, vb, Ob, Lb = (a[cu[b]:cu[b + 1]] for a in (q, k, v, O, LSE))
        plain = np.array([where[("prefix", i)] for i in range(P)] + [where[("draft", t)] for t in range(T)])
        L = len(plain)
        qr, kr = rope_complex(qb[plain], np.arange(L), w.rope_theta), rope_complex(kb[plain], np.arange(L), w.rope_theta)
        ref = library_causal(qr, kr, vb[plain], G, scale)
        worst = max(worst, float(np.abs(ref - Ob[plain]).max()))
        worst = max(worst, float(np.abs(library_causal_lse(qr, kr, G, scale) - Lb[plain]).max()))
        for kk in range(K):
            own = np.array([where[("suffix", kk, a)] for a in range(S)])
            idx = np.r_[plain[:P + bounds[kk]], own]
            L = len(idx)
            qr, kr = rope_complex(qb[idx], np.arange(L), w.rope_theta), rope_complex(kb[idx], np.arange(L), w.rope_theta)
            ref = library_causal(qr, kr, vb[idx], G, scale)
            worst = max(worst, float(np.abs(ref[-S:] - Ob[own]).max()))
            worst = max(worst, float(np.abs(library_causal_lse(qr, kr, G, scale)[-S:] - Lb[own]).max()))
    assert worst < atol, worst


def test_standalone_equivalence_interleaved():
    pr = wl.Problem([3, 0, 7], [20, 9, 33], [3, 2, 0], [5, 1, 4], [[0, 7, 20], [4, 4], []], layout=1)
    standalone_check(wl.make_custom(pr, 6, 2, 64, dtype=torch.float32, rope_theta=1e4, seed=21))
    t = wl.make("tiny", rope_theta=5e5).problem
    pr = wl.Problem(t.prompt_len, t.draft_len, t.num_segments, t.segment_len, t.boundaries, layout=1)
    standalone_check(wl.make_custom(pr, 2, 1, 64, dtype=torch.float32, rope_theta=5e5, seed=22))


def test_attention_is_the_appended_result_reordered():
    P, T, S, bounds = 5, 40, 3, [4, 17, 17, 33]
    pr = wl.Problem([P], [T], [len(bounds)], [S], [bounds])
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.float32, rope_theta=5e5, seed=23)
    perm = to_appended(P, T, S, bounds)
    q, k, v = (x.double().numpy() for x in (w.q, w.k, w.v))
    OA, LA = orc.masked_attention([P], [T], [len(bounds)], [S], [bounds], q, k, v, rope_theta=5e5, return_lse=True)
    qB, kB, vB = (np.empty_like(x) for x in (q, k, v))
    qB[perm], kB[perm], vB[perm] = q, k, v          # the same tokens, packed the other way
    OB, LB = orc.masked_attention([P], [T], [len(bounds)], [S], [bounds], qB, kB, vB, rope_theta=5e5,
                                  return_lse=True, layout=orc.LAYOUT_INTERLEAVED)
    assert np.abs(OB[perm] - OA).max() < 1e-12 and np.abs(LB[perm] - LA).max() < 1e-12
