"""The whole step (pv_build_mask, pv_masked_attention, pv_first_reject, then the segment-only call) under
HIP graph capture: the library allocates nothing, never synchronises and takes the plan's host image by
value, so a captured step must replay to the bits of the eager step.  The graph is replayed several times
with eager work and synchronisations in between, and every replay is checked."""
import numpy as np
import pytest
import torch

import pv_workloads as wl
from oracle import pv_oracle as orc
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")


def test_captured_step_replays_bit_exact():
    pr = wl.Problem([64, 3], [448, 70], [8, 2], [32, 5], [[32, 64, 100, 128, 200, 300, 447, 448], [9, 70]])
    w = wl.make_custom(pr, 8, 2, 128, dtype=torch.bfloat16, rope_theta=5e5, seed=5)
    ver = gc.make_verifier(pv, w)
    dev = ver.device
    q, k, v, logits = w.q.to(dev), w.k.to(dev), w.v.to(dev), w.logits.to(dev)
    thr = orc.margin_threshold(w.tau)
    out = torch.empty_like(q)
    out_seg = torch.zeros_like(q)

    def step():
        ver.build_mask()
        ver.attention(q, k, v, out=out, rope_theta=w.rope_theta)
        ver.first_reject(logits, thr, 0)
        ver.segment_attention(q, k, v, out_seg, rope_theta=w.rope_theta)

    ver.plan.zero_()                                  # alignment gaps of the plan are never written
    step()                                            # eager: also the library's one-time device check
    torch.cuda.synchronize()
    want = (out.clone(), ver.readout.clone(), out_seg.clone(), ver.plan.clone())

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        # eager work between the replays: scribble over every output, then replay
        out.fill_(1.0); out_seg.fill_(0.0); ver.readout.fill_(-7); ver.plan.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), want[0].view(torch.int16)), rep
        assert torch.equal(ver.readout, want[1]), rep
        seg_rows = torch.from_numpy(np.concatenate([
            np.arange(64 + 448, 64 + 448 + 8 * 32), 768 + np.arange(3 + 70, 3 + 70 + 2 * 5)])).to(dev)
        assert torch.equal(out_seg[seg_rows].view(torch.int16), want[2][seg_rows].view(torch.int16)), rep
        assert torch.equal(ver.plan, want[3]), rep


def test_captured_prepared_fp8_and_static_calls_replay_bit_exact():
    # the calls added beside the three of the step: prepared keys (dense), the segment rows over them, the
    # FP8 K/V pass and the pass with the library's own workspace, captured together and replayed
    pr = wl.Problem([64, 3], [448, 70], [8, 2], [32, 5], [[32, 64, 100, 128, 200, 300, 447, 448], [9, 70]])
    w = wl.make_custom(pr, 8, 2, 128, dtype=torch.bfloat16, rope_theta=5e5, seed=6)
    ver = gc.make_verifier(pv, w)
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    kc, ksc = (t.to(dev) for t in wl.quantize_fp8(w.k))
    vc, vsc = (t.to(dev) for t in wl.quantize_fp8(w.v))
    ws2 = torch.empty_like(ver.workspace)
    out_seg, out_fp8, out_static = torch.zeros_like(q), torch.zeros_like(q), torch.zeros_like(q)

    def calls():
        ver.build_mask()
        pv.pv_prepare_kv(ver.sizes, ver.plan, k, v, ws2, rope_theta=w.rope_theta)
        pv.pv_segment_attention_prepared(ver.sizes, ver.plan, q, k, v, out_seg, ws2, rope_theta=w.rope_theta)
        pv.pv_masked_attention_fp8kv(ver.sizes, ver.plan, q, kc, vc, ksc, vsc, out_fp8, ver.workspace,
                                     rope_theta=w.rope_theta)
        pv.pv_masked_attention_static(ver.sizes, ver.plan, q, k, v, out_static, rope_theta=w.rope_theta)

    calls()                                           # eager: also the one-time device queries of the library
    torch.cuda.synchronize()
    seg_rows = torch.from_numpy(np.concatenate([
        np.arange(64 + 448, 64 + 448 + 8 * 32), 768 + np.arange(3 + 70, 3 + 70 + 2 * 5)])).to(dev)
    want = (out_seg[seg_rows].clone(), out_fp8.clone(), out_static.clone())
    # the static-workspace pass is the ordinary pass, bit for bit
    assert torch.equal(out_static.view(torch.int16), ver.attention(q, k, v, rope_theta=w.rope_theta).view(torch.int16))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    for rep in range(3):
        out_seg.fill_(0.0); out_fp8.fill_(1.0); out_static.fill_(2.0); ws2.fill_(0); ver.plan.fill_(0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_seg[seg_rows].view(torch.int16), want[0].view(torch.int16)), rep
        assert torch.equal(out_fp8.view(torch.int16), want[1].view(torch.int16)), rep
        assert torch.equal(out_static.view(torch.int16), want[2].view(torch.int16)), rep
