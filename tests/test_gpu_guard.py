"""Guard regions: every buffer the library writes (plan, dense mask, workspace, out, lse, readout,
judge logits, decision) sits inside a larger allocation filled with a pattern; after the whole step and
the follow-up calls every guard byte must still hold it.  All kernels run normally: nothing is
provoked, the test only looks at what the launches left around their outputs."""
import ctypes as C
import dataclasses

import numpy as np
import pytest
import torch

import pv_workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")

GUARD = 4096          # bytes on either side; a multiple of every alignment the library asks for
PATTERN = 0xA5


class Guarded:
    """`nbytes` usable bytes between two guard regions, viewed as `dtype`."""
    def __init__(self, nbytes, dtype, dev, shape=None):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 16
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), PATTERN, dtype=torch.uint8, device=dev)
        self.body = self.raw[GUARD:GUARD + self.nbytes].view(dtype)
        if shape is not None:
            self.body = self.body.view(*shape)

    def intact(self):
        front = self.raw[:GUARD]
        back = self.raw[GUARD + self.nbytes:]
        return bool((front == PATTERN).all()) and bool((back == PATTERN).all())


def run_guarded(pr, hq, hkv, d, theta, dense=True):
    w = wl.make_custom(pr, hq, hkv, d, dtype=torch.bfloat16, rope_theta=theta, seed=77)
    dev = gc.device()
    prob = pv.make_problem(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len,
                           pr.flat_boundaries(), pr.layout)
    sz = pv.pv_query_sizes(prob, hq, hkv, d, pv.PV_BF16)
    n, ns, B = sz.total_tokens, sz.total_segments, sz.batch
    hs = 256
    bufs = {
        "plan": Guarded(sz.plan_bytes, torch.int32, dev),
        "workspace": Guarded(sz.attn_workspace_bytes, torch.uint8, dev),
        "out_bf16": Guarded(n * hq * d * 2, torch.bfloat16, dev, (n, hq, d)),
        "out_f32": Guarded(n * hq * d * 4, torch.float32, dev, (n, hq, d)),
        "out_seg": Guarded(n * hq * d * 2, torch.bfloat16, dev, (n, hq, d)),
        "lse": Guarded(hq * n * 4, torch.float32, dev, (hq, n)),
        "readout": Guarded(B * 4 * 4, torch.int32, dev, (B, 4)),
        "decision": Guarded(B * 12 * 4, torch.int32, dev, (B, 12)),
        "logits": Guarded(max(ns, 1) * 2 * 4, torch.float32, dev, (max(ns, 1), 2)),
        "exported": Guarded(4 * n * 4, torch.int32, dev),
    }
    if dense:
        bufs["dense_mask"] = Guarded(sz.dense_mask_bytes, torch.uint8, dev)
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    hidden = torch.randn(n, hs, device=dev).bfloat16()
    w2 = torch.randn(2, hs, device=dev).bfloat16()
    full_lg = torch.zeros(B, 2, device=dev)
    thr = pv.pv_margin_from_tau(0.9)
    pol = pv.make_policy(thr, 1.0, 5.0, 2.0, [2.0, 2.0], 0.3, 2, 0.0)
    plan, ws = bufs["plan"].body, bufs["workspace"].body
    pv.pv_build_mask(prob, sz, plan, bufs["dense_mask"].body if dense else None)
    pv.pv_masked_attention(sz, plan, q, k, v, bufs["out_bf16"].body, ws, bufs["lse"].body, rope_theta=theta)
    pv.pv_masked_attention(sz, plan, q, k, v, bufs["out_f32"].body, ws, None, rope_theta=theta)
    pv.pv_segment_attention(sz, plan, q, k, v, bufs["out_seg"].body, ws, bufs["lse"].body, rope_theta=theta)
    logits = bufs["logits"].body[:ns]
    pv.pv_judge_logits(sz, plan, hidden, w2, logits)
    pv.pv_first_reject(sz, plan, logits, thr, 0, bufs["readout"].body)
    pv.pv_decide(sz, plan, logits, full_lg, pol, bufs["decision"].body)
    ex = bufs["exported"].body

    st = pv.lib.pv_plan_export(C.byref(sz), plan.data_ptr(), ex[:n].data_ptr(), ex[n:2 * n].data_ptr(),
                               ex[2 * n:3 * n].data_ptr(), ex[3 * n:3 * n + max(ns, 1)].data_ptr() if ns else None,
                               torch.cuda.current_stream().cuda_stream)
    assert st == pv.PV_OK
    torch.cuda.synchronize()
    for name, g in bufs.items():
        assert g.intact(), name
    # the calls did write: the bodies no longer hold the pattern everywhere
    assert not bool((bufs["out_bf16"].raw[GUARD:GUARD + 64] == PATTERN).all())
    assert bool(torch.isfinite(bufs["out_f32"].body).all())


EDGE = [
    (wl.Problem([0], [1], [0], [1], [[]]), 4, 1, 128, 5e5),
    (wl.Problem([0], [7], [3], [1], [[0, 0, 7]]), 4, 2, 128, 5e5),
    (wl.Problem([5], [64], [4], [5], [[1, 33, 64, 64]]), 8, 2, 128, 5e5),
    (wl.Problem([31], [97], [2], [33], [[50, 97]]), 5, 1, 128, 0.0),
    (wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
                [[0, 7, 20], [4, 4], [], [32, 64]]), 16, 2, 128, 1e4),
    (wl.Problem([100], [300], [1], [70], [[300]]), 6, 2, 64, 5e5),
    (wl.Problem([17], [200], [6], [16], [[0, 10, 64, 65, 128, 200]]), 3, 1, 64, 1e4),
    (wl.Problem([40], [300], [5], [24], [[17, 90, 91, 200, 300]]), 7, 1, 128, 5e5),
]


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("idx", range(len(EDGE)))
def test_guards_edge_shapes(idx, layout):
    pr, hq, hkv, d, theta = EDGE[idx]
    run_guarded(dataclasses.replace(pr, layout=layout), hq, hkv, d, theta)


@pytest.mark.parametrize("layout", [0, 1])
def test_guards_ragged_batch(layout):
    # the ragged configuration (16 requests, the multi-kernel plan), without its 250 MB dense mask
    pr = dataclasses.replace(wl.make("ragged").problem, layout=layout)
    run_guarded(pr, 32, 8, 128, 5e5, dense=False)
