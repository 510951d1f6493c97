"""GPU parity of the fp32 debug path of pv_masked_attention (max-abs <= 1e-5 vs the fp64 oracle)."""
import numpy as np
import pytest
import torch

import pv_workloads as wl
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")

TOL_F32 = 1e-5


def check(w, softmax_scale=0.0):
    out, lse = gc.run_gpu_attention(pv, w, lse=True, softmax_scale=softmax_scale)
    ref, ref_lse = gc.oracle_attention(w, return_lse=True, scale=softmax_scale or None)
    err = np.abs(out.double().cpu().numpy() - ref)
    assert err.max() <= TOL_F32, err.max()
    lerr = np.abs(lse.double().cpu().numpy().T - ref_lse)
    assert lerr.max() <= 1e-4, lerr.max()


def test_tiny():
    check(wl.make("tiny"))


def test_tiny_with_rope():
    check(wl.make("tiny", rope_theta=5e5))


@pytest.mark.parametrize("d,hq,hkv", [(64, 6, 2), (128, 5, 1)])
def test_ragged_small_f32(d, hq, hkv):
    pr = wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
                    [[0, 7, 20], [4, 4], [], [32, 64]])
    check(wl.make_custom(pr, hq, hkv, d, dtype=torch.float32, rope_theta=1e4, seed=21, value_scale=0.5))


@pytest.mark.parametrize("theta", [0.0, 5e5])
@pytest.mark.parametrize("scale", [0.05, 0.2])
def test_softmax_scale_f32(scale, theta):
    pr = wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
                    [[0, 7, 20], [4, 4], [], [32, 64]])
    check(wl.make_custom(pr, 6, 2, 64, dtype=torch.float32, rope_theta=theta, seed=31, value_scale=0.5),
          softmax_scale=scale)
