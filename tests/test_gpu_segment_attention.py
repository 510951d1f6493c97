"""GPU parity of pv_segment_attention (segment rows only, long work items split along the keys and
merged) against the fp64 oracle, through the C ABI.  Same tolerances as the full pass (bf16 inputs:
max-abs 1e-2, mean-abs 1e-3 on the fp32-output run; the bf16-output run within half a bf16 ulp
more); every row that is not a segment row must keep the bits it had before the call."""
import dataclasses

import numpy as np
import pytest
import torch

import pv_workloads as wl
from tests import gpu_common as gc
from tests.test_gpu_attention_bf16 import check_errors

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")


def segment_rows(pr):
    """Per request the local rows of its segment tokens, in the caller's row order."""
    from oracle import pv_oracle as orc
    rows = []
    for b in range(pr.batch):
        P, T, K, S = pr.prompt_len[b], pr.draft_len[b], pr.num_segments[b], pr.segment_len[b]
        if pr.layout == 1:
            toks = orc.interleaved_tokens(P, T, S, pr.boundaries[b])
            rows.append([i for i, t in enumerate(toks) if t[0] == 'e'])
        else:
            rows.append(list(range(P + T, P + T + K * S)))
    return rows


def check_segments(w, sample=None, seed=0):
    pr = w.problem
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    rows = segment_rows(pr)
    if sample is not None:
        rng = np.random.default_rng(seed)
        rows = [sorted(set(int(x) for x in rng.choice(r, size=min(sample, len(r)), replace=False))) if r else []
                for r in rows]
    all_seg = torch.from_numpy(gc.packed_row_index(pr, segment_rows(pr))).to(dev) if pr.total_segments else None
    ref, ref_lse = gc.oracle_attention(w, rows_per_request=rows, return_lse=True)
    idx = torch.from_numpy(gc.packed_row_index(pr, rows)).to(dev)
    outs = {}
    for dt in (torch.float32, torch.bfloat16):
        out = torch.full(q.shape, 7.25, dtype=dt, device=dev)          # sentinel: must survive elsewhere
        lse = torch.full((w.n_q_heads, pr.total_tokens), -3.5, dtype=torch.float32, device=dev)
        ver.segment_attention(q, k, v, out, lse=lse, rope_theta=w.rope_theta)
        torch.cuda.synchronize()
        keep = torch.ones(pr.total_tokens, dtype=torch.bool, device=dev)
        if all_seg is not None:
            keep[all_seg] = False
        assert bool((out[keep] == 7.25).all()) and bool((lse[:, keep] == -3.5).all())
        if len(idx):
            check_errors(out.index_select(0, idx).double().cpu().numpy(), ref, bf16_out=dt == torch.bfloat16)
            lerr = np.abs(lse.index_select(1, idx).double().cpu().numpy().T - ref_lse)
            assert lerr.max() <= 1e-2, lerr.max()
        outs[dt] = out
    # the same rows from the full pass.  The pieces round their probabilities to bf16 against their
    # own reference, so the two calls differ by rounding of the size the tolerance allows, no more
    full = gc.run_gpu_attention(pv, w, out_dtype=torch.float32, ver=ver)
    if all_seg is not None and len(all_seg):
        d = (full.index_select(0, all_seg) - outs[torch.float32].index_select(0, all_seg)).abs()
        assert d.max().item() <= 1e-2 and d.mean().item() <= 1e-3, (d.max().item(), d.mean().item())
    return ver


PROBLEMS = [
    wl.Problem([0], [7], [3], [1], [[0, 0, 7]]),
    wl.Problem([5], [64], [4], [5], [[1, 33, 64, 64]]),
    wl.Problem([31], [97], [2], [33], [[50, 97]]),
    wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
               [[0, 7, 20], [4, 4], [], [32, 64]]),
    wl.Problem([100], [300], [1], [70], [[300]]),
    wl.Problem([64], [448], [8], [32], [[32, 64, 100, 128, 200, 300, 447, 448]]),
    wl.Problem([40], [900], [5], [24], [[17, 90, 91, 500, 900]]),
    wl.Problem([9], [30], [0], [4], [[]]),                                   # no segment at all: nothing written
]


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("idx", range(len(PROBLEMS)))
def test_small_problems(idx, layout):
    pr = dataclasses.replace(PROBLEMS[idx], layout=layout)
    group, d = [(4, 128), (1, 64), (3, 128), (8, 64), (5, 128)][idx % 5]
    w = wl.make_custom(pr, group * 2, 2, d, dtype=torch.bfloat16, rope_theta=5e5 if idx % 2 else 0.0, seed=80 + idx)
    ver = check_segments(w)
    assert ver.sizes.n_seg_tiles == sum(
        (pr.seq_len(b) + 31) // 32 - (pr.prompt_len[b] + pr.draft_len[b]) // 32 if pr.num_segments[b] else 0
        for b in range(pr.batch))


def test_8b_all_segment_rows():
    check_segments(wl.make("8b"))


def test_8b_interleaved():
    w = wl.make("8b")
    check_segments(wl.Workload(**{**w.__dict__, "problem": dataclasses.replace(w.problem, layout=1)}))


def test_14b_sampled():
    check_segments(wl.make("14b"), sample=96)


def test_ragged_sampled():
    check_segments(wl.make("ragged"), sample=12)


def test_70b_sampled():
    check_segments(wl.make("70b"), sample=24)
