"""Pins for the oracle's mask, positions and judge rows (CPU only).

None of these re-type the oracle's rule: they use (a) the stand-alone-run reading of
"Parallel Prefix Verification" (every token's visible set is the context of the sequence
it would belong to if its prefix were judged alone), built with Python sets on tiny cases;
(b) closed-form counts; (c) special cases that collapse to a textbook causal mask.
"""
import itertools

import numpy as np
import pytest

from oracle import pv_oracle as orc
import pv_workloads as wl


def standalone_context(P, T, S, bounds, i):
    """Token indices (in the packed layout) that token i would have in its context if
    the pair (prompt + draft[:p_k], suffix) were run on its own -- including i itself."""
    if i < P + T:
        return list(range(i + 1))
    k, a = divmod(i - P - T, S)
    start = P + T + k * S
    return list(range(P)) + list(range(P, P + bounds[k])) + list(range(start, start + a + 1))


def nondecreasing_tuples(T, K):
    return itertools.combinations_with_replacement(range(T + 1), K)


def test_mask_and_positions_exhaustive_tiny():
    checked = 0
    for P in (0, 1, 2):
        for T in (1, 3, 6):
            for K in (0, 1, 2, 3):
                for S in (1, 2, 3):
                    if K == 0 and S > 1:
                        continue
                    for bounds in nondecreasing_tuples(T, K):
                        N = P + T + K * S
                        M = orc.dense_mask(P, T, S, bounds)
                        pos = orc.positions(P, T, S, bounds)
                        assert M.shape == (N, N) and M.dtype == np.uint8
                        for i in range(N):
                            ctx = standalone_context(P, T, S, bounds, i)
                            expect = np.zeros(N, dtype=np.uint8)
                            expect[ctx] = 1
                            assert np.array_equal(M[i], expect), (P, T, K, S, bounds, i)
                            # position = index of the token inside its stand-alone sequence
                            assert pos[i] == len(ctx) - 1
                        checked += 1
    assert checked > 500


@pytest.mark.parametrize("name", ["tiny", "8b"])
def test_mask_closed_form_counts(name):
    w = wl.make(name)
    pr = w.problem
    P, T, K, S = pr.prompt_len[0], pr.draft_len[0], pr.num_segments[0], pr.segment_len[0]
    b = pr.boundaries[0]
    N = pr.seq_len(0)
    assert N == P + T + K * S                      # "one prefill of length T + n*|suffix|" (+ prompt)
    M = orc.dense_mask(P, T, S, b)
    total = (P + T) * (P + T + 1) // 2 + sum(S * (P + p) + S * (S + 1) // 2 for p in b)
    assert int(M.sum(dtype=np.int64)) == total
    # row sums: causal rows see i+1 keys; row a of segment k sees P + p_k + a + 1
    rs = M.sum(axis=1, dtype=np.int64)
    assert np.array_equal(rs[:P + T], np.arange(1, P + T + 1))
    for k in range(K):
        for a in range(S):
            assert rs[P + T + k * S + a] == P + b[k] + a + 1
    # invariants
    assert np.all(np.diag(M) == 1)
    assert np.all(np.triu(M[:P + T, :P + T], 1) == 0)
    assert np.all(M[:P + T, P + T:] == 0)
    for k in range(K):
        r0 = P + T + k * S
        blk = M[r0:r0 + S]
        assert np.all(blk[:, :P + b[k]] == 1)
        assert np.all(blk[:, P + b[k]:P + T] == 0)
        assert np.array_equal(blk[:, r0:r0 + S], np.tril(np.ones((S, S), dtype=np.uint8)))
        other = np.ones(N, dtype=bool)
        other[:P + T] = False
        other[r0:r0 + S] = False
        assert np.all(blk[:, other] == 0)          # copies never see each other


def test_mask_special_cases_reduce_to_causal():
    # no segments: plain lower-triangular mask
    M = orc.dense_mask(5, 9, 1, [])
    assert np.array_equal(M, np.tril(np.ones((14, 14), dtype=np.uint8)))
    assert np.array_equal(orc.positions(5, 9, 1, []), np.arange(14))
    # one segment that sees the whole draft: the packed sequence IS a plain causal sequence
    M = orc.dense_mask(4, 7, 3, [7])
    assert np.array_equal(M, np.tril(np.ones((14, 14), dtype=np.uint8)))
    assert np.array_equal(orc.positions(4, 7, 3, [7]), np.arange(14))


def test_mask_row_subset_matches_full():
    w = wl.make("tiny")
    pr = w.problem
    args = (pr.prompt_len[0], pr.draft_len[0], pr.segment_len[0], pr.boundaries[0])
    full = orc.dense_mask(*args)
    rows = [0, 31, 32, 287, 288, 303, 304, 351]
    assert np.array_equal(orc.dense_mask(*args, rows=rows), full[rows])


def test_judge_rows_are_last_token_of_each_segment():
    P, T, S, K = 3, 10, 4, 5
    jr = orc.judge_rows(P, T, S, K)
    assert list(jr) == [P + T + S - 1 + S * k for k in range(K)]
    assert jr[-1] == P + T + K * S - 1


def test_workload_structure_is_valid():
    for name in ("tiny", "8b", "ragged", "14b"):
        w = wl.make(name)
        pr = w.problem
        for b in range(pr.batch):
            bs = pr.boundaries[b]
            assert len(bs) == pr.num_segments[b]
            assert all(0 <= x <= pr.draft_len[b] for x in bs)
            assert all(bs[i] <= bs[i + 1] for i in range(len(bs) - 1))
        assert w.q.shape == (pr.total_tokens, w.n_q_heads, w.head_dim)
        assert w.k.shape == (pr.total_tokens, w.n_kv_heads, w.head_dim)
        assert w.logits.shape == (pr.total_segments, 2)
    # determinism of the seeded generator
    a, b = wl.make("8b"), wl.make("8b")
    assert a.problem.boundaries == b.problem.boundaries
    assert bool((a.q.view(dtype=__import__("torch").int16) == b.q.view(dtype=__import__("torch").int16)).all())
