"""GPU parity of the interleaved packing (every segment directly after the draft tokens it judges,
appendix "Parallel partial verify") against the oracle's interleaved functions, through the C ABI:
dense mask, positions and judge rows bit-exact; attention within the tolerances of the appended
layout (bf16: max-abs 1e-2, mean-abs 1e-3; fp32 path 1e-5); and, because both layouts hold the same
tokens, the bf16 result must be the appended layout's result reordered, bit for bit."""
import dataclasses

import numpy as np
import pytest
import torch

import pv_workloads as wl
from oracle import pv_oracle as orc
from tests import gpu_common as gc
from tests.test_gpu_attention_bf16 import check_full, check_sampled

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")


def inter(pr):
    return dataclasses.replace(pr, layout=1)


PROBLEMS = [
    wl.Problem([0], [1], [0], [1], [[]]),
    wl.Problem([0], [7], [3], [1], [[0, 0, 7]]),
    wl.Problem([5], [64], [4], [5], [[1, 33, 64, 64]]),
    wl.Problem([31], [97], [2], [33], [[50, 97]]),
    wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
               [[0, 7, 20], [4, 4], [], [32, 64]]),
    wl.Problem([100], [300], [1], [70], [[150]]),
    wl.Problem([40], [300], [5], [24], [[17, 90, 91, 200, 300]]),
]


@pytest.mark.parametrize("idx", range(len(PROBLEMS)))
def test_plan_bit_exact(idx):
    pr = inter(PROBLEMS[idx])
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.float32, seed=1)
    ver = gc.make_verifier(pv, w, dense_mask=True)
    ver.build_mask()
    pos, ae, bs, jr = pv.pv_plan_export(ver.sizes, ver.plan)
    torch.cuda.synchronize()
    assert np.array_equal(ver.dense_mask.cpu().numpy(), gc.oracle_dense_mask_flat(pr))
    opos, ojr = gc.oracle_plan_arrays(pr)
    assert np.array_equal(pos.cpu().numpy().astype(np.int64), opos)
    assert np.array_equal(jr.cpu().numpy().astype(np.int64), ojr)


@pytest.mark.parametrize("idx", range(len(PROBLEMS)))
def test_attention_fp32_path(idx):
    pr = inter(PROBLEMS[idx])
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.float32, rope_theta=5e5, seed=40 + idx)
    out, lse = gc.run_gpu_attention(pv, w, lse=True)
    ref, ref_lse = gc.oracle_attention(w, return_lse=True)
    assert np.abs(out.double().cpu().numpy() - ref).max() <= 1e-5
    assert np.abs(lse.double().cpu().numpy().T - ref_lse).max() <= 1e-4


@pytest.mark.parametrize("idx", range(len(PROBLEMS)))
def test_attention_bf16(idx):
    pr = inter(PROBLEMS[idx])
    group, d = [(4, 128), (1, 64), (3, 128), (8, 64)][idx % 4]
    w = wl.make_custom(pr, group * 2, 2, d, dtype=torch.bfloat16, rope_theta=5e5 if idx % 2 else 0.0, seed=60 + idx)
    check_full(w)


def interleaved_8b():
    w = wl.make("8b")
    return wl.Workload(**{**w.__dict__, "problem": inter(w.problem)})


def test_8b_interleaved_full():
    check_full(interleaved_8b())


def test_ragged_interleaved_sampled():
    w = wl.make("ragged")
    check_sampled(wl.Workload(**{**w.__dict__, "problem": inter(w.problem)}), n_random=32)


def test_same_tokens_give_the_appended_result_reordered():
    # q/k/v of the interleaved run are the appended run's rows moved to where the interleaved
    # packing puts them; the kernels then do the same arithmetic in the same order
    w = wl.make("8b")
    pr = w.problem
    verA = gc.make_verifier(pv, w); verA.build_mask()
    outA = gc.run_gpu_attention(pv, w, ver=verA)
    wB = interleaved_8b()
    verB = gc.make_verifier(pv, wB); verB.build_mask()
    # where each row of the appended order goes: the judge rows and positions of both plans agree
    # on it, but build it from the oracle's token list to stay independent of the library
    toks = orc.interleaved_tokens(pr.prompt_len[0], pr.draft_len[0], pr.segment_len[0], pr.boundaries[0])
    P, T, S = pr.prompt_len[0], pr.draft_len[0], pr.segment_len[0]
    perm = np.empty(len(toks), dtype=np.int64)
    for row, t in enumerate(toks):
        src = t[1] if t[0] == 'q' else (P + t[2] if t[0] == 'c' else P + T + t[1] * S + t[2])
        perm[src] = row
    idx = torch.from_numpy(perm)
    q, k, v = (torch.empty_like(x) for x in (w.q, w.k, w.v))
    q[idx], k[idx], v[idx] = w.q, w.k, w.v
    wB = wl.Workload(**{**wB.__dict__, "q": q, "k": k, "v": v})
    outB = gc.run_gpu_attention(pv, wB, ver=verB)
    assert torch.equal(outB[idx.to(outB.device)].view(torch.int16), outA.view(torch.int16))


def test_readout_and_judge_gather_use_the_interleaved_judge_rows():
    pr = inter(PROBLEMS[4])
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.bfloat16, seed=3)
    ver = gc.make_verifier(pv, w); ver.build_mask()
    H = 256
    gen = torch.Generator().manual_seed(5)
    hidden = torch.randn(pr.total_tokens, H, generator=gen).bfloat16()
    w2 = (torch.randn(2, H, generator=gen) * 0.1).bfloat16()
    got = ver.judge_logits(hidden.cuda(), w2.cuda()).cpu().numpy()
    _, ojr = gc.oracle_plan_arrays(pr)
    ref = orc.judge_logits(hidden.double().numpy(), w2.double().numpy(), ojr)
    assert np.abs(got - ref).max() <= 1e-5 * float(np.abs(hidden.double().numpy()[ojr][:, None, :] * w2.double().numpy()[None]).sum(-1).max())
    thr = orc.margin_threshold(w.tau)
    fr = ver.first_reject(w.logits.cuda(), thr, 0).cpu().numpy()
    assert np.array_equal(fr, orc.first_reject(w.logits.numpy(), pr.num_segments, pr.boundaries, thr, 0))
