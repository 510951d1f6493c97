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


# ---------------------------------------------------------------- prepared keys, paged K/V

def _run_unsplit(ver, w, q, k, v, dtype):
    out = torch.full(q.shape, 7.25, dtype=dtype, device=q.device)
    lse = torch.full((w.n_q_heads, w.problem.total_tokens), -3.5, dtype=torch.float32, device=q.device)
    ver.segment_attention(q, k, v, out, lse=lse, rope_theta=w.rope_theta)
    torch.cuda.synchronize()
    return out, lse


def _same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("idx", [0, 1, 3, 5, 6])
def test_prepared_keys_equal_the_unsplit_call(idx, layout):
    # pv_prepare_kv + pv_segment_attention_prepared against pv_segment_attention: bit for bit, dense K/V
    # and K/V scattered over a page pool through a block table
    pr = dataclasses.replace(PROBLEMS[idx], layout=layout)
    group, d = [(4, 128), (1, 64), (3, 128), (8, 64), (5, 128)][idx % 5]
    w = wl.make_custom(pr, group * 2, 2, d, dtype=torch.bfloat16, rope_theta=5e5 if idx % 2 else 0.0, seed=180 + idx)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    n = pr.total_tokens
    for dtype in (torch.float32, torch.bfloat16):
        want, want_lse = _run_unsplit(ver, w, q, k, v, dtype)
        # dense
        ws = torch.full_like(ver.workspace, 0x5A)
        pv.pv_prepare_kv(ver.sizes, ver.plan, k, v, ws, rope_theta=w.rope_theta)
        out = torch.full(q.shape, 7.25, dtype=dtype, device=dev)
        lse = torch.full_like(want_lse, -3.5)
        pv.pv_segment_attention_prepared(ver.sizes, ver.plan, q, k, v, out, ws, lse, rope_theta=w.rope_theta)
        torch.cuda.synchronize()
        assert _same_bits(out, want) and _same_bits(lse, want_lse)
        # a second judge pass over the same prepared keys (nothing re-prepared): the same bits again
        out.fill_(7.25); lse.fill_(-3.5)
        pv.pv_segment_attention_prepared(ver.sizes, ver.plan, q, k, v, out, ws, lse, rope_theta=w.rope_theta)
        torch.cuda.synchronize()
        assert _same_bits(out, want) and _same_bits(lse, want_lse)
        # paged: pages of 16 tokens in a shuffled pool with spare pages
        ps = 16
        n_pages = (n + ps - 1) // ps
        rng = np.random.default_rng(idx)
        table = torch.from_numpy(rng.permutation(n_pages + 3)[:n_pages].astype(np.int32)).to(dev)
        pool_k = torch.full(((n_pages + 3) * ps, w.n_kv_heads, d), float("nan"), dtype=torch.bfloat16, device=dev)
        pool_v = torch.full_like(pool_k, float("nan"))
        rows = torch.arange(n, device=dev)
        dst = table.long()[rows // ps] * ps + rows % ps
        pool_k[dst] = k
        pool_v[dst] = v
        ws2 = torch.full_like(ver.workspace, 0x33)
        pv.pv_prepare_kv(ver.sizes, ver.plan, pool_k, pool_v, ws2, rope_theta=w.rope_theta, block_table=table, page_size=ps)
        out.fill_(7.25); lse.fill_(-3.5)
        pv.pv_segment_attention_prepared(ver.sizes, ver.plan, q, pool_k, pool_v, out, ws2, lse, rope_theta=w.rope_theta,
                                         block_table=table, page_size=ps)
        torch.cuda.synchronize()
        assert _same_bits(out, want) and _same_bits(lse, want_lse)


def test_prepared_keys_survive_a_grown_draft():
    # Premature verification at T_p draft tokens, then the pass over the finished draft (appendix "Full
    # pipeline", Stage 1 and Stage 4): the second pass prepares only the tokens from P + T_p on and must
    # give the bits of a call that prepares everything; both are checked against the oracle.
    P, Tp, T, S = 70, 300, 700, 8
    early = wl.Problem([P], [Tp], [3], [S], [[100, 200, 300]])
    late = wl.Problem([P], [T], [6], [S], [[100, 200, 300, 450, 600, 700]])
    wB = wl.make_custom(late, 8, 2, 128, dtype=torch.bfloat16, rope_theta=5e5, seed=210)
    wA = wl.make_custom(early, 8, 2, 128, dtype=torch.bfloat16, rope_theta=5e5, seed=211)
    # the early pass sees the same prompt and the first T_p draft tokens
    for name in ("q", "k", "v"):
        getattr(wA, name)[:P + Tp] = getattr(wB, name)[:P + Tp]
    verA, verB = gc.make_verifier(pv, wA), gc.make_verifier(pv, wB)
    verA.build_mask(); verB.build_mask()
    dev = verB.device
    cap = verB.sizes.padded_keys
    nbytes = max(pv.pv_prepared_workspace_bytes(verA.sizes, cap), pv.pv_prepared_workspace_bytes(verB.sizes, cap))
    ws = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device=dev)
    qA, kA, vA = wA.q.to(dev), wA.k.to(dev), wA.v.to(dev)
    qB, kB, vB = wB.q.to(dev), wB.k.to(dev), wB.v.to(dev)
    # early pass
    pv.pv_prepare_kv(verA.sizes, verA.plan, kA, vA, ws, rope_theta=5e5, key_capacity=cap)
    outA = torch.zeros(qA.shape, dtype=torch.float32, device=dev)
    pv.pv_segment_attention_prepared(verA.sizes, verA.plan, qA, kA, vA, outA, ws, rope_theta=5e5, key_capacity=cap)
    torch.cuda.synchronize()
    rowsA = segment_rows(early)
    check_errors(outA[rowsA[0]].double().cpu().numpy(), gc.oracle_attention(wA, rows_per_request=rowsA), bf16_out=False)
    # late pass: only the new tokens are prepared
    pv.pv_prepare_kv(verB.sizes, verB.plan, kB, vB, ws, rope_theta=5e5, first_token=P + Tp, key_capacity=cap)
    outB = torch.zeros(qB.shape, dtype=torch.float32, device=dev)
    lseB = torch.zeros(wB.n_q_heads, late.total_tokens, dtype=torch.float32, device=dev)
    pv.pv_segment_attention_prepared(verB.sizes, verB.plan, qB, kB, vB, outB, ws, lseB, rope_theta=5e5, key_capacity=cap)
    torch.cuda.synchronize()
    want, want_lse = _run_unsplit(verB, wB, qB, kB, vB, torch.float32)
    rowsB = segment_rows(late)
    idx = torch.tensor(rowsB[0], device=dev)
    assert _same_bits(outB[idx], want[idx]) and _same_bits(lseB[:, idx], want_lse[:, idx])
    check_errors(outB[idx].double().cpu().numpy(), gc.oracle_attention(wB, rows_per_request=rowsB), bf16_out=False)


def test_prepared_8b_and_argument_checks():
    w = wl.make("8b")
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    want, want_lse = _run_unsplit(ver, w, q, k, v, torch.bfloat16)
    pv.pv_prepare_kv(ver.sizes, ver.plan, k, v, ver.workspace, rope_theta=w.rope_theta)
    out = torch.full(q.shape, 7.25, dtype=torch.bfloat16, device=dev)
    lse = torch.full_like(want_lse, -3.5)
    pv.pv_segment_attention_prepared(ver.sizes, ver.plan, q, k, v, out, ver.workspace, lse, rope_theta=w.rope_theta)
    torch.cuda.synchronize()
    assert _same_bits(out, want) and _same_bits(lse, want_lse)
    for bad in (dict(first_token=-1), dict(first_token=5, last_token=4), dict(last_token=w.problem.total_tokens + 1),
                dict(key_capacity=ver.sizes.padded_keys - 64), dict(key_capacity=ver.sizes.padded_keys + 1),
                dict(block_table=torch.zeros(4, dtype=torch.int32, device=dev), page_size=0)):
        with pytest.raises(pv.PvError) as e:
            pv.pv_prepare_kv(ver.sizes, ver.plan, k, v, ver.workspace, rope_theta=w.rope_theta, **bad)
        assert e.value.status == pv.PV_ERR_SHAPE, bad


# The rows with very few visible keys are evaluated in fp32 by one piece of code in two places: extra
# workgroups of the main kernel's launch in a whole pass (rotary angles read from the table), blocks of
# the preparation launch in the segment-only call (angles computed on the spot).  Segment rows that see
# almost nothing must come out of both with the same bits.
@pytest.mark.parametrize("d,group", [(128, 4), (128, 8), (64, 4), (128, 5)])
def test_short_segment_rows_same_bits_in_both_calls(d, group):
    pr = wl.Problem([0, 3], [40, 9], [4, 2], [6, 20], [[0, 1, 2, 40], [0, 5]])
    w = wl.make_custom(pr, 2 * group, 2, d, dtype=torch.bfloat16, rope_theta=5e5, seed=4242 + d + group)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    assert ver.sizes.n_short_seg_rows > 0
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    seg = torch.from_numpy(gc.packed_row_index(pr, segment_rows(pr))).to(dev)
    for dt in (torch.float32, torch.bfloat16):
        full = torch.zeros(q.shape, dtype=dt, device=dev)
        lse_full = torch.zeros((w.n_q_heads, pr.total_tokens), dtype=torch.float32, device=dev)
        ver.attention(q, k, v, out=full, lse=lse_full, rope_theta=w.rope_theta)
        only = torch.zeros(q.shape, dtype=dt, device=dev)
        lse_only = torch.zeros((w.n_q_heads, pr.total_tokens), dtype=torch.float32, device=dev)
        ver.segment_attention(q, k, v, only, lse=lse_only, rope_theta=w.rope_theta)
        torch.cuda.synchronize()
        a, b = full.index_select(0, seg), only.index_select(0, seg)
        la, lb = lse_full.index_select(1, seg), lse_only.index_select(1, seg)
        # at least the segment rows that the plan lists as short must agree bit for bit
        plan_short = ver.sizes.n_short_seg_rows
        same_rows = (a.view(a.shape[0], -1) == b.view(b.shape[0], -1)).all(dim=1)
        assert int(same_rows.sum()) >= plan_short, (int(same_rows.sum()), plan_short)
        same_lse = (la == lb).all(dim=0)
        assert int(same_lse.sum()) >= plan_short
