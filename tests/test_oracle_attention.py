"""Pins for the oracle's rotary embedding and masked attention (CPU only).

The main pin is the independence statement of "Parallel Prefix Verification": the rows of
suffix copy k must equal what a stand-alone causal pass over [prompt, draft[:p_k], copy k]
produces, with positions 0..len-1.  The stand-alone pass uses a library attention
(torch scaled_dot_product_attention, is_causal=True, fp64) and a rotary embedding written
with complex multiplication, so it shares no formula with the oracle.
"""
import math

import numpy as np
import pytest
import torch

from oracle import pv_oracle as orc
import pv_workloads as wl


def rope_complex(x, pos, theta):
    """Rotary embedding as a complex rotation: (x_c + i x_{c+D/2}) * exp(i * pos * theta^(-2c/D))."""
    if theta == 0.0:
        return x.copy()
    D = x.shape[-1]
    z = x[..., :D // 2] + 1j * x[..., D // 2:]
    w = np.array([theta ** (-(2.0 * c) / D) for c in range(D // 2)])
    rot = np.exp(1j * np.asarray(pos, dtype=np.float64)[:, None] * w[None, :])[:, None, :]
    y = z * rot
    return np.concatenate([y.real, y.imag], axis=-1)


def library_causal(q, k, v, G, scale):
    """torch SDPA (fp64, causal) on [L, H, D] arrays; GQA by repeating kv heads."""
    tq = torch.from_numpy(q).permute(1, 0, 2).unsqueeze(0)
    tk = torch.from_numpy(np.repeat(k, G, axis=1)).permute(1, 0, 2).unsqueeze(0)
    tv = torch.from_numpy(np.repeat(v, G, axis=1)).permute(1, 0, 2).unsqueeze(0)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


def library_causal_lse(q, k, G, scale):
    """Natural-log softmax normaliser of every row of a stand-alone causal pass, [L, Hq]: library
    matmul, library lower-triangular fill, torch.logsumexp (fp64)."""
    tq = torch.from_numpy(q).permute(1, 0, 2)
    tk = torch.from_numpy(np.repeat(k, G, axis=1)).permute(1, 0, 2)
    s = torch.matmul(tq, tk.transpose(1, 2)) * scale                    # [Hq, L, L]
    L = s.shape[-1]
    s = s.masked_fill(~torch.ones(L, L, dtype=torch.bool).tril(), float("-inf"))
    return torch.logsumexp(s, dim=-1).transpose(0, 1).numpy()


def standalone_check(w, atol=1e-11):
    pr = w.problem
    G = w.n_q_heads // w.n_kv_heads
    scale = 1.0 / math.sqrt(w.head_dim)
    q = w.q.double().numpy(); k = w.k.double().numpy(); v = w.v.double().numpy()
    O, LSE = orc.masked_attention(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len,
                                  pr.boundaries, q, k, v, rope_theta=w.rope_theta, return_lse=True)
    cu = pr.token_offsets()
    worst = 0.0
    for b in range(pr.batch):
        P, T, K, S = pr.prompt_len[b], pr.draft_len[b], pr.num_segments[b], pr.segment_len[b]
        qb, kb, vb, Ob, Lb = (a[cu[b]:cu[b + 1]] for a in (q, k, v, O, LSE))
        # prompt + draft alone: appending suffix copies changes nothing for them
        L = P + T
        qr, kr = rope_complex(qb[:L], np.arange(L), w.rope_theta), rope_complex(kb[:L], np.arange(L), w.rope_theta)
        ref = library_causal(qr, kr, vb[:L], G, scale)
        worst = max(worst, float(np.abs(ref - Ob[:L]).max()))
        worst = max(worst, float(np.abs(library_causal_lse(qr, kr, G, scale) - Lb[:L]).max()))
        for kk in range(K):
            p = pr.boundaries[b][kk]
            seg = slice(P + T + kk * S, P + T + (kk + 1) * S)
            idx = np.r_[0:P + p, seg]
            L = len(idx)
            qr, kr = rope_complex(qb[idx], np.arange(L), w.rope_theta), rope_complex(kb[idx], np.arange(L), w.rope_theta)
            ref = library_causal(qr, kr, vb[idx], G, scale)
            worst = max(worst, float(np.abs(ref[-S:] - Ob[seg]).max()))
            worst = max(worst, float(np.abs(library_causal_lse(qr, kr, G, scale)[-S:] - Lb[seg]).max()))
    assert worst < atol, worst
    return worst


def test_standalone_equivalence_tiny():
    standalone_check(wl.make("tiny"))


def test_standalone_equivalence_tiny_with_rope():
    standalone_check(wl.make("tiny", rope_theta=5e5))


def test_standalone_equivalence_gqa_ragged_small():
    pr = wl.Problem([3, 0, 7], [20, 9, 33], [3, 2, 0], [5, 1, 4], [[0, 7, 20], [4, 4], []])
    w = wl.make_custom(pr, 6, 2, 64, dtype=torch.float32, rope_theta=1e4, seed=11)
    standalone_check(w)
    w = wl.make_custom(pr, 5, 1, 128, dtype=torch.bfloat16, rope_theta=5e5, seed=12)
    standalone_check(w)


def test_rope_properties():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(7, 2, 8))
    pos = np.array([0, 1, 2, 3, 50, 1000, 14335])
    y = orc.rope(x, pos, 5e5)
    assert np.array_equal(y[0], x[0])                                  # position 0 = identity
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=0, atol=1e-12)
    assert np.allclose(y, rope_complex(x, pos, 5e5), rtol=0, atol=1e-12)
    # D = 2: a plain planar rotation by `pos` radians (inverse frequency 1)
    e = np.array([[[1.0, 0.0]]])
    r = orc.rope(e, np.array([3]), 10.0)
    assert np.allclose(r[0, 0], [math.cos(3.0), math.sin(3.0)], atol=1e-15)
    # scores depend only on relative position
    q = rng.normal(size=(1, 1, 16)); k = rng.normal(size=(1, 1, 16))
    s1 = (orc.rope(q, np.array([40]), 1e4) * orc.rope(k, np.array([33]), 1e4)).sum()
    s2 = (orc.rope(q, np.array([1007]), 1e4) * orc.rope(k, np.array([1000]), 1e4)).sum()
    assert abs(s1 - s2) < 1e-12
    # theta = 0 disables the rotation
    assert np.array_equal(orc.rope(x, pos, 0.0), x)


def test_isolation_and_permutation_metamorphic():
    w = wl.make("tiny", rope_theta=5e5)
    pr = w.problem
    P, T, K, S = pr.prompt_len[0], pr.draft_len[0], pr.num_segments[0], pr.segment_len[0]
    b = pr.boundaries[0]
    q = w.q.double().numpy(); k = w.k.double().numpy(); v = w.v.double().numpy()
    run = lambda kk, vv, bb=b, qq=q: orc.masked_attention([P], [T], [len(bb)], [S], [bb], qq, kk, vv, 5e5)
    base = run(k, v)
    # perturb every other copy and every draft token beyond the boundary of copy 1
    k2, v2 = k.copy(), v.copy()
    seg1 = slice(P + T + S, P + T + 2 * S)
    for other in (0, 2, 3):
        sl = slice(P + T + other * S, P + T + (other + 1) * S)
        k2[sl] += 3.0; v2[sl] -= 2.0
    k2[P + b[1]:P + T] *= -1.5; v2[P + b[1]:P + T] += 7.0
    pert = run(k2, v2)
    assert np.array_equal(pert[seg1], base[seg1])                      # bit-identical
    assert not np.array_equal(pert[P + T - 1], base[P + T - 1])        # the perturbation was real
    # permuting the copies (with their boundaries) permutes the outputs
    perm = [2, 0, 3, 1]
    take = np.r_[0:P + T, np.concatenate([np.arange(P + T + s * S, P + T + (s + 1) * S) for s in perm])]
    outp = orc.masked_attention([P], [T], [K], [S], [[b[s] for s in perm]], q[take], k[take], v[take], 5e5)
    assert np.allclose(outp, base[take], rtol=0, atol=1e-13)


def test_constant_values_and_lse():
    pr = wl.Problem([4], [12], [2], [3], [[5, 12]])
    w = wl.make_custom(pr, 2, 1, 64, dtype=torch.float32, seed=3)
    q = w.q.double().numpy(); k = w.k.double().numpy()
    v = np.full(k.shape, 0.625)
    O, lse = orc.masked_attention([4], [12], [2], [3], [[5, 12]], q, k, v, return_lse=True)
    assert np.allclose(O, 0.625, rtol=0, atol=1e-14)                   # convex combination
    # the first token attends only to itself: lse = its own scaled score
    s00 = (q[0, :, :] * k[0, 0, :][None, :]).sum(-1) / 8.0
    assert np.allclose(lse[0], s00, atol=1e-13)
    # all positions zero (theta irrelevant): same as no rotation at position 0 everywhere
    a = orc.attention(q, k, v, orc.dense_mask(4, 12, 3, [5, 12]))
    assert np.allclose(a, O, atol=1e-14)


def test_lse_closed_forms_and_scale():
    # all keys identical: every visible score is the same s, so lse = s + ln(number of visible keys)
    P, T, S, bounds = 3, 9, 2, [4, 9]
    N = P + T + 2 * S
    rng = np.random.default_rng(8)
    q = rng.normal(size=(N, 2, 8))
    k = np.tile(rng.normal(size=(1, 1, 8)), (N, 1, 1))
    v = rng.normal(size=(N, 1, 8))
    M = orc.dense_mask(P, T, S, bounds)
    for scale in (None, 0.05, 0.7):
        sc = (1.0 / math.sqrt(8)) if scale is None else scale
        O, lse = orc.attention(q, k, v, M, scale=scale, return_lse=True)
        s = (q * k).sum(-1) * sc                                         # [N, 2]
        count = M.sum(axis=1).astype(np.float64)                         # visible keys per row
        assert np.allclose(lse, s + np.log(count)[:, None], rtol=0, atol=1e-13)
        # identical scores: O is the plain mean of the visible V rows
        want = (M.astype(np.float64) @ v[:, 0, :]) / count[:, None]
        assert np.allclose(O[:, 0], want, rtol=0, atol=1e-13) and np.allclose(O[:, 1], want, rtol=0, atol=1e-13)
    # a non-default scale is the default one applied to queries stretched by the ratio
    w = wl.make_custom(wl.Problem([4], [12], [2], [3], [[5, 12]]), 2, 1, 64, dtype=torch.float32, seed=9)
    qq, kk, vv = (x.double().numpy() for x in (w.q, w.k, w.v))
    a = orc.masked_attention([4], [12], [2], [3], [[5, 12]], qq, kk, vv, scale=0.2, return_lse=True)
    b = orc.masked_attention([4], [12], [2], [3], [[5, 12]], qq * (0.2 * 8.0), kk, vv, return_lse=True)
    assert np.allclose(a[0], b[0], rtol=0, atol=1e-13) and np.allclose(a[1], b[1], rtol=0, atol=1e-13)


@pytest.mark.parametrize("rows", [[0, 5, 17, 21]])
def test_row_subset_matches_full(rows):
    pr = wl.Problem([4], [12], [2], [3], [[5, 12]])
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.bfloat16, rope_theta=5e5, seed=5)
    q = w.q.double().numpy(); k = w.k.double().numpy(); v = w.v.double().numpy()
    full = orc.masked_attention([4], [12], [2], [3], [[5, 12]], q, k, v, 5e5)
    sub = orc.masked_attention([4], [12], [2], [3], [[5, 12]], q, k, v, 5e5, rows_per_request=[rows])
    assert np.allclose(sub, full[rows], rtol=0, atol=1e-14)
