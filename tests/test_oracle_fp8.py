"""Pins for the oracle's FP8 K/V reading (CPU only): the E4M3 decoder against a library conversion
and the format's defining values, and the attention against stand-alone library passes over the
de-quantised tensors in which only Q is rotated."""
import math

import numpy as np
import torch

from oracle import pv_oracle as orc
import pv_workloads as wl
from tests.test_oracle_attention import library_causal, library_causal_lse, rope_complex


def test_decoder_all_codes():
    codes = np.arange(256, dtype=np.uint8)
    got = orc.decode_e4m3(codes)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).double().numpy()        # library conversion
    assert np.array_equal(np.isnan(got), np.isnan(lib)) and np.isnan(got).sum() == 2  # 0x7F and 0xFF only
    ok = ~np.isnan(lib)
    assert np.array_equal(got[ok], lib[ok])
    # defining values of the format: largest 448, smallest normal 2^-6, smallest subnormal 2^-9, 1.0 = 0x38
    assert got[0x7E] == 448.0 and got[0xFE] == -448.0
    assert got[0x08] == 2.0 ** -6 and got[0x01] == 2.0 ** -9 and got[0x38] == 1.0
    assert got[0x00] == 0.0 and got[0x80] == 0.0 and np.signbit(got[0x80])
    # monotone over the positive codes, and symmetric
    assert (np.diff(got[0:0x7F]) > 0).all()
    assert np.array_equal(got[0x80:0xFF], -got[0x00:0x7F])


def standalone_check_fp8(w, atol=1e-11):
    pr = w.problem
    G = w.n_q_heads // w.n_kv_heads
    scale = 1.0 / math.sqrt(w.head_dim)
    kc, ksc = wl.quantize_fp8(w.k)
    vc, vsc = wl.quantize_fp8(w.v)
    q = w.q.double().numpy()
    O, LSE = orc.masked_attention_fp8kv(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len,
                                        pr.boundaries, q, kc.numpy(), vc.numpy(), ksc.numpy(), vsc.numpy(),
                                        rope_theta=w.rope_theta, return_lse=True)
    # de-quantised tensors through the library: codes -> float8 tensor -> double, times the scale
    k = kc.view(torch.float8_e4m3fn).double().numpy() * ksc.double().numpy()[None, :, None]
    v = vc.view(torch.float8_e4m3fn).double().numpy() * vsc.double().numpy()[None, :, None]
    cu = pr.token_offsets()
    worst = 0.0
    for b in range(pr.batch):
        P, T, K, S = pr.prompt_len[b], pr.draft_len[b], pr.num_segments[b], pr.segment_len[b]
        qb, kb, vb, Ob, Lb = (a[cu[b]:cu[b + 1]] for a in (q, k, v, O, LSE))
        L = P + T
        qr = rope_complex(qb[:L], np.arange(L), w.rope_theta)            # keys are NOT rotated
        worst = max(worst, float(np.abs(library_causal(qr, kb[:L], vb[:L], G, scale) - Ob[:L]).max()))
        worst = max(worst, float(np.abs(library_causal_lse(qr, kb[:L], G, scale) - Lb[:L]).max()))
        for kk in range(K):
            p = pr.boundaries[b][kk]
            seg = slice(P + T + kk * S, P + T + (kk + 1) * S)
            idx = np.r_[0:P + p, seg]
            L = len(idx)
            qr = rope_complex(qb[idx], np.arange(L), w.rope_theta)
            worst = max(worst, float(np.abs(library_causal(qr, kb[idx], vb[idx], G, scale)[-S:] - Ob[seg]).max()))
            worst = max(worst, float(np.abs(library_causal_lse(qr, kb[idx], G, scale)[-S:] - Lb[seg]).max()))
    assert worst < atol, worst


def test_standalone_equivalence_fp8kv():
    pr = wl.Problem([3, 0, 7], [20, 9, 33], [3, 2, 0], [5, 1, 4], [[0, 7, 20], [4, 4], []])
    standalone_check_fp8(wl.make_custom(pr, 6, 2, 64, dtype=torch.bfloat16, rope_theta=1e4, seed=41))
    standalone_check_fp8(wl.make_custom(pr, 5, 1, 128, dtype=torch.bfloat16, rope_theta=0.0, seed=42))
    t = wl.make("tiny", rope_theta=5e5)
    standalone_check_fp8(wl.make_custom(t.problem, 2, 1, 64, dtype=torch.bfloat16, rope_theta=5e5, seed=43))


def test_scales_and_rotation_of_q_only():
    pr = wl.Problem([4], [12], [2], [3], [[5, 12]])
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.bfloat16, rope_theta=5e5, seed=44)
    kc, ksc = wl.quantize_fp8(w.k)
    vc, vsc = wl.quantize_fp8(w.v)
    args = ([4], [12], [2], [3], [[5, 12]], w.q.double().numpy(), kc.numpy(), vc.numpy())
    base = orc.masked_attention_fp8kv(*args, ksc.numpy(), vsc.numpy(), rope_theta=5e5)
    # V scale is linear in the output; a K scale is a softmax scale
    twice = orc.masked_attention_fp8kv(*args, ksc.numpy(), 2 * vsc.numpy(), rope_theta=5e5)
    assert np.allclose(twice, 2 * base, rtol=0, atol=1e-13)
    a = orc.masked_attention_fp8kv(*args, 4 * ksc.numpy(), vsc.numpy(), rope_theta=5e5)      # exact in fp32
    b = orc.masked_attention_fp8kv(*args, ksc.numpy(), vsc.numpy(), rope_theta=5e5, scale=4.0 / 8.0)
    assert np.allclose(a, b, rtol=0, atol=1e-13)
    # exactly representable K and V (small integers, scale 1): the plain pass with unrotated keys
    rng = np.random.default_rng(0)
    ki = torch.from_numpy(rng.integers(-8, 9, size=w.k.shape).astype(np.float32))
    vi = torch.from_numpy(rng.integers(-8, 9, size=w.v.shape).astype(np.float32))
    kci, vci = ki.to(torch.float8_e4m3fn).view(torch.uint8).numpy(), vi.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    one = np.ones(2, dtype=np.float32)
    got = orc.masked_attention_fp8kv([4], [12], [2], [3], [[5, 12]], w.q.double().numpy(), kci, vci, one, one, rope_theta=5e5)
    pos = orc.positions(4, 12, 3, [5, 12])
    qr = orc.rope(w.q.double().numpy(), pos, 5e5)
    want = orc.attention(qr, ki.double().numpy(), vi.double().numpy(), orc.dense_mask(4, 12, 3, [5, 12]))
    assert np.allclose(got, want, rtol=0, atol=1e-13)
    # rotating the keys as well would be a different result (the reading matters)
    other = orc.attention(qr, orc.rope(ki.double().numpy(), pos, 5e5), vi.double().numpy(), orc.dense_mask(4, 12, 3, [5, 12]))
    assert np.abs(other - want).max() > 1e-3
