"""pv_masked_attention_static (the entry point for callers that cannot allocate: its workspace is a
fixed array inside the library) against pv_masked_attention, through the C ABI: two calls in a row, the
second on a smaller problem, each bit-identical to the ordinary call and within the tolerance of the
oracle; then a problem beyond the fixed size, which must be refused before anything is launched."""
import ctypes as C

import numpy as np
import pytest
import torch

import pv_workloads as wl
from tests import gpu_common as gc
from tests.test_gpu_attention_bf16 import check_errors

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")


def both_calls(w):
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    n, hq = w.problem.total_tokens, w.n_q_heads
    assert pv.pv_static_workspace_needed(ver.sizes) <= pv.PV_STATIC_WORKSPACE_BYTES
    res = {}
    for name in ("ordinary", "static"):
        out = torch.full(q.shape, 3.0, dtype=torch.float32, device=dev)
        lse = torch.full((hq, n), -1.0, dtype=torch.float32, device=dev)
        args = (C.byref(ver.sizes), ver.plan.data_ptr(), q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                lse.data_ptr(), pv.PV_F32, 0.0, w.rope_theta)
        stream = torch.cuda.current_stream().cuda_stream
        if name == "ordinary":
            st = pv.lib.pv_masked_attention(*args, ver.workspace.data_ptr(), ver.workspace.numel(), stream)
        else:
            st = pv.lib.pv_masked_attention_static(*args, stream)
        assert st == pv.PV_OK, (name, st)
        torch.cuda.synchronize()
        res[name] = (out, lse)
    assert torch.equal(res["ordinary"][0].view(torch.int32), res["static"][0].view(torch.int32))
    assert torch.equal(res["ordinary"][1].view(torch.int32), res["static"][1].view(torch.int32))
    return res["static"][0]


def test_static_workspace_two_calls_then_too_large():
    # first call: the 8B-like configuration (14 MB of workspace); second: a small ragged batch that
    # reuses the front of the same array with the first call's bytes still behind it
    big = wl.make("8b")
    out = both_calls(big)
    rows = gc.sample_rows(big.problem, n_random=64, seed=1)
    ref = gc.oracle_attention(big, rows_per_request=rows)
    idx = torch.from_numpy(gc.packed_row_index(big.problem, rows)).to(out.device)
    check_errors(out.index_select(0, idx).double().cpu().numpy(), ref, bf16_out=False)
    small = wl.make_custom(wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
                                      [[0, 7, 20], [4, 4], [], [32, 64]]), 16, 2, 128,
                           dtype=torch.bfloat16, rope_theta=1e4, seed=104)
    out = both_calls(small)
    check_errors(out.double().cpu().numpy(), gc.oracle_attention(small), bf16_out=False)
    # beyond the fixed size: refused with PV_ERR_WORKSPACE, nothing launched, outputs untouched
    wr = wl.make("ragged")
    ver = gc.make_verifier(pv, wr)
    assert pv.pv_static_workspace_needed(ver.sizes) > pv.PV_STATIC_WORKSPACE_BYTES
    ver.build_mask()
    dev = ver.device
    q, k, v = wr.q.to(dev), wr.k.to(dev), wr.v.to(dev)
    o = torch.full(q.shape, 3.0, dtype=torch.float32, device=dev)
    with pytest.raises(pv.PvError) as e:
        pv.pv_masked_attention_static(ver.sizes, ver.plan, q, k, v, o)
    assert e.value.status == pv.PV_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((o == 3.0).all())
