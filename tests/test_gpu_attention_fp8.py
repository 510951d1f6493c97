"""GPU parity of pv_masked_attention_fp8kv (K and V as FP8 E4M3 codes with a scale per kv head, both
products on the FP8 matrix instruction) against the fp64 oracle on the same codes.

Tolerance.  The oracle takes K and V exactly as stored.  Q goes through the FP8 pipe as two E4M3 terms
(rounded value plus scaled residual), which leaves it at about bf16 precision; what remains is the
rounding of the probabilities to E4M3: 3 mantissa bits, relative error up to 2^-4, uniform, standard
deviation 2^-4 / sqrt(3) = 3.6 %.  The output is a weighted mean of V rows whose weights are each off
by that much at random (the row sum is taken over the rounded weights, so they still sum to one): for
V ~ N(0,1) the error of an output has standard deviation 0.036 / sqrt(n_eff), n_eff = 1 / sum p_j^2 the
number of keys that carry the weight.  Rows just above the fp32 short-row limit (n_eff about 20) give
8e-3, and ten of those deviations bound the tail of the 10^7 outputs of a configuration: max-abs 8e-2.
The mean over rows whose n_eff runs from tens to thousands stays below 5e-3, and the normaliser, a
log of the same perturbed sum, below 5e-2.  Measured: max-abs 1.9e-2 (70b) to 5.9e-2 (14b, outlier
channels), mean-abs 6e-4 to 2.8e-3, normaliser 1e-2 to 3.2e-2.  The bf16 path's 1e-2 / 1e-3 are not
claimed for this storage format.  Rows with at most PV_SHORT_ROW_KEYS keys are evaluated in fp32 and
must meet 1e-4."""
import dataclasses

import numpy as np
import pytest
import torch

import pv_workloads as wl
from oracle import pv_oracle as orc
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")

MAX_ABS, MEAN_ABS, LSE_ABS = 8e-2, 5e-3, 5e-2


def run_fp8(w, out_dtype=torch.float32, rows=None, label=None):
    pr = w.problem
    kc, ksc = wl.quantize_fp8(w.k)
    vc, vsc = wl.quantize_fp8(w.v)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    dev = ver.device
    q = w.q.to(dev)
    out = torch.full(q.shape, 5.5, dtype=out_dtype, device=dev)
    lse = torch.zeros(w.n_q_heads, pr.total_tokens, dtype=torch.float32, device=dev)
    pv.pv_masked_attention_fp8kv(ver.sizes, ver.plan, q, kc.to(dev), vc.to(dev), ksc.to(dev), vsc.to(dev), out,
                                 ver.workspace, lse, rope_theta=w.rope_theta)
    torch.cuda.synchronize()
    ref, ref_lse = orc.masked_attention_fp8kv(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len,
                                              pr.boundaries, w.q.double().numpy(), kc.numpy(), vc.numpy(),
                                              ksc.numpy(), vsc.numpy(), rope_theta=w.rope_theta,
                                              rows_per_request=rows, return_lse=True, layout=pr.layout)
    if rows is not None:
        idx = torch.from_numpy(gc.packed_row_index(pr, rows)).to(dev)
        got, got_lse = out.index_select(0, idx), lse.index_select(1, idx)
    else:
        got, got_lse = out, lse
    got = got.double().cpu().numpy()
    assert np.isfinite(got).all()
    err = np.abs(got - ref)
    lerr = np.abs(got_lse.double().cpu().numpy().T - ref_lse)
    if label:
        print(f"[fp8kv {label}] max_abs={err.max():.3e} mean_abs={err.mean():.3e} lse max_abs={lerr.max():.3e} "
              f"max|O|={np.abs(ref).max():.3f}", flush=True)
    half_ulp = 0.0 if out_dtype == torch.float32 else 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -126))) - 8)
    assert (err <= MAX_ABS + half_ulp).all(), err.max()
    assert err.mean() <= MEAN_ABS, err.mean()
    assert lerr.max() <= LSE_ABS, lerr.max()
    return out, ref, ver


EDGE = [
    (wl.Problem([0], [1], [0], [1], [[]]), 4, 1, 5e5),
    (wl.Problem([0], [7], [3], [1], [[0, 0, 7]]), 4, 2, 5e5),
    (wl.Problem([5], [64], [4], [5], [[1, 33, 64, 64]]), 8, 2, 5e5),
    (wl.Problem([31], [97], [2], [33], [[50, 97]]), 5, 1, 0.0),
    (wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
                [[0, 7, 20], [4, 4], [], [32, 64]]), 16, 2, 1e4),
    (wl.Problem([64], [448], [8], [32], [[32, 64, 100, 128, 200, 300, 447, 448]]), 2, 2, 5e5),
    (wl.Problem([40], [300], [5], [24], [[17, 90, 91, 200, 300]]), 7, 1, 5e5),
]


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("idx", range(len(EDGE)))
def test_edge_cases(idx, layout):
    pr, hq, hkv, theta = EDGE[idx]
    w = wl.make_custom(dataclasses.replace(pr, layout=layout), hq, hkv, 128, dtype=torch.bfloat16,
                       rope_theta=theta, seed=600 + idx)
    out32, ref, ver = run_fp8(w, label=f"edge {idx} layout {layout}")
    out16, _, _ = run_fp8(w, out_dtype=torch.bfloat16)
    assert torch.equal(out32.to(torch.bfloat16).view(torch.int16), out16.view(torch.int16))   # same kernel, RNE at the end
    # rows with few keys come from the fp32 evaluation
    short = []
    cu = pr.token_offsets()
    M = gc.oracle_dense_mask_flat(w.problem)
    off = 0
    for b in range(pr.batch):
        n = pr.seq_len(b)
        cnt = M[off:off + n * n].reshape(n, n).sum(axis=1)
        short += [cu[b] + int(i) for i in np.nonzero(cnt <= 16)[0]]
        off += n * n
    if short:
        e = np.abs(out32[short].double().cpu().numpy() - ref[short])
        assert e.max() <= 1e-4, e.max()


@pytest.mark.parametrize("group", [1, 2, 3, 4, 5, 6, 7, 8])
def test_group_sizes_long_rows(group):
    pr = wl.Problem([70], [850], [3], [40], [[333, 600, 850]])
    w = wl.make_custom(pr, group, 1, 128, dtype=torch.bfloat16, rope_theta=5e5 if group % 2 else 0.0, seed=640 + group)
    run_fp8(w, label=f"group {group}")


def test_8b_every_row():
    run_fp8(wl.make("8b"), label="8b, every row")


def test_14b_sampled():
    w = wl.make("14b")
    run_fp8(w, rows=gc.sample_rows(w.problem, n_random=128, seed=w.seed), label="14b, sampled rows")


def test_70b_sampled():
    w = wl.make("70b")
    run_fp8(w, rows=gc.sample_rows(w.problem, n_random=64, seed=w.seed), label="70b, sampled rows")


def test_refuses_other_head_sizes_and_fp32_queries():
    pr = wl.Problem([5], [64], [2], [5], [[33, 64]])
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.bfloat16, seed=1)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    dev = ver.device
    kc, ksc = wl.quantize_fp8(w.k)
    out = torch.zeros_like(w.q).to(dev)
    with pytest.raises(pv.PvError) as e:
        pv.pv_masked_attention_fp8kv(ver.sizes, ver.plan, w.q.to(dev), kc.to(dev), kc.to(dev), ksc.to(dev),
                                     ksc.to(dev), out, ver.workspace)
    assert e.value.status == pv.PV_ERR_SHAPE
    torch.cuda.synchronize()
