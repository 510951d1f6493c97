"""GPU parity (bit-exact): pv_build_mask's dense mask, positions, judge rows and
pv_first_reject against the oracle, through the C ABI."""
import itertools

import numpy as np
import pytest
import torch

import pv_workloads as wl
from oracle import pv_oracle as orc
from tests import gpu_common as gc

pytestmark = pytest.mark.gpu
pv = pytest.importorskip("paper_2605_04263_amd.binding")

EDGE_PROBLEMS = [
    wl.Problem([0], [1], [0], [1], [[]]),                                  # smallest: one token
    wl.Problem([0], [7], [3], [1], [[0, 0, 7]]),                           # no prompt, p=0, duplicate
    wl.Problem([5], [64], [4], [5], [[1, 33, 64, 64]]),                    # S=5 like a chat suffix
    wl.Problem([31], [97], [2], [33], [[50, 97]]),                         # ragged vs 32/64 tiles
    wl.Problem([3, 0, 7, 64], [20, 9, 33, 64], [3, 2, 0, 2], [5, 1, 4, 32],
               [[0, 7, 20], [4, 4], [], [32, 64]]),                        # ragged batch with K=0
    wl.Problem([100], [300], [1], [70], [[300]]),                          # K=1, p=T: plain causal
]


def check_plan(pr, hq=4, hkv=2, d=64, dtype=torch.float32):
    w = wl.make_custom(pr, hq, hkv, d, dtype=dtype, seed=1)
    ver = gc.make_verifier(pv, w, dense_mask=True)
    ver.build_mask()
    pos, ae, bs, jr = pv.pv_plan_export(ver.sizes, ver.plan)
    torch.cuda.synchronize()
    assert ver.sizes.total_tokens == pr.total_tokens
    assert np.array_equal(ver.dense_mask.cpu().numpy(), gc.oracle_dense_mask_flat(pr))
    opos, ojr = gc.oracle_plan_arrays(pr)
    assert np.array_equal(pos.cpu().numpy().astype(np.int64), opos)
    assert np.array_equal(jr.cpu().numpy().astype(np.int64), ojr)
    return ver


@pytest.mark.parametrize("idx", range(len(EDGE_PROBLEMS)))
def test_mask_edge_cases(idx):
    check_plan(EDGE_PROBLEMS[idx])


@pytest.mark.parametrize("name", ["tiny", "8b", "14b"])
def test_mask_named_configs(name):
    w = wl.make(name)
    check_plan(w.problem, w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)


def test_mask_ragged_config_rows_sampled():
    # full dense mask of the ragged batch is ~250 MB: compare it whole on the GPU side per request
    w = wl.make("ragged")
    pr = w.problem
    ver = gc.make_verifier(pv, w, dense_mask=True)
    ver.build_mask()
    torch.cuda.synchronize()
    off = 0
    for b in range(pr.batch):
        n = pr.seq_len(b)
        got = ver.dense_mask[off:off + n * n].cpu().numpy().reshape(n, n)
        exp = orc.dense_mask(pr.prompt_len[b], pr.draft_len[b], pr.segment_len[b], pr.boundaries[b])
        assert np.array_equal(got, exp), b
        off += n * n


def test_readout_named_and_patterns():
    for name in ("tiny", "8b", "ragged", "14b"):
        w = wl.make(name)
        pr = w.problem
        ver = gc.make_verifier(pv, w)
        ver.build_mask()
        lg = w.logits.to(ver.device)
        for tau in (0.5, 0.88, 0.985, 0.998):
            thr = orc.margin_threshold(tau)
            for mode in (0, 1):
                got = ver.first_reject(lg, thr, mode).cpu().numpy()
                exp = orc.first_reject(w.logits.numpy(), pr.num_segments, pr.boundaries, thr, mode)
                assert np.array_equal(got, exp), (name, tau, mode)


def test_70b_plan_mask_work_list_readout():
    # the long configuration (4 requests of 14 336 tokens, 1 792 tiles: the plan comes from the separate
    # upload / tokens / tiles / ranking kernels): positions and judge rows of every token, the dense
    # mask of every request entry by entry (822 MB on the device, one request at a time on the host),
    # the row descriptors (rebuilt into mask rows), the tile classifier and the order of the work
    # list against the oracle's mask, and the readout in both modes
    w = wl.make("70b")
    pr = w.problem
    ver = gc.make_verifier(pv, w, dense_mask=True)
    ver.build_mask()
    pos, ae, bs, jr = pv.pv_plan_export(ver.sizes, ver.plan)
    torch.cuda.synchronize()
    assert ver.sizes.total_tokens == pr.total_tokens == 57344 and ver.sizes.total_segments == 256
    opos, ojr = gc.oracle_plan_arrays(pr)
    assert np.array_equal(pos.cpu().numpy().astype(np.int64), opos)
    assert np.array_equal(jr.cpu().numpy().astype(np.int64), ojr)
    tiles, work = _work_list(ver)
    ae_h, bs_h = ae.cpu().numpy(), bs.cpu().numpy()
    cu = pr.token_offsets()
    off, t = 0, 0
    for b in range(pr.batch):
        n = pr.seq_len(b)
        print(f"70b request {b}: oracle mask", flush=True)
        M = orc.dense_mask(pr.prompt_len[b], pr.draft_len[b], pr.segment_len[b], pr.boundaries[b])
        got = ver.dense_mask[off:off + n * n].cpu().numpy().reshape(n, n)
        assert np.array_equal(got, M), b
        del got
        # key j is visible to row i iff j < a_end or b_start <= j <= i: sampled rows of the request
        j = np.arange(n)
        for i in gc.sample_rows(pr, n_random=64, seed=b)[b]:
            a, s0 = int(ae_h[cu[b] + i]), int(bs_h[cu[b] + i])
            assert np.array_equal(((j < a) | ((j >= s0) & (j <= i))).astype(np.uint8), M[i]), (b, i)
        t = check_tiles_of_request(tiles, t, cu[b], M)
        del M
        off += n * n
    assert t == len(tiles) == 1792
    check_work_order(tiles, work)
    lg = w.logits.to(ver.device)
    for tau in (0.5, 0.88, 0.985, 0.998):
        thr = orc.margin_threshold(tau)
        for mode in (0, 1):
            got = ver.first_reject(lg, thr, mode).cpu().numpy()
            exp = orc.first_reject(w.logits.numpy(), pr.num_segments, pr.boundaries, thr, mode)
            assert np.array_equal(got, exp), (tau, mode)


def test_readout_all_patterns_k6_batched():
    K = 6
    pats = list(itertools.product([0, 1], repeat=K))
    B = len(pats)
    bounds = [[2, 5, 5, 9, 14, 20]] * B
    pr = wl.Problem([3] * B, [20] * B, [K] * B, [2] * B, bounds)
    w = wl.make_custom(pr, 1, 1, 64, dtype=torch.float32, seed=2)
    rng = np.random.default_rng(0)
    lg = np.zeros((B * K, 2), np.float32)
    for b, p in enumerate(pats):
        for k, c in enumerate(p):
            m = rng.uniform(2.0, 6.0) if c else rng.uniform(-6.0, 1.9)
            base = rng.normal()
            lg[b * K + k] = (base + m, base)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    for mode in (0, 1):
        got = ver.first_reject(torch.from_numpy(lg).to(ver.device), 2.0, mode).cpu().numpy()
        exp = orc.first_reject(lg, pr.num_segments, pr.boundaries, 2.0, mode)
        assert np.array_equal(got, exp)


def test_readout_ties_and_k0():
    pr = wl.Problem([2, 2], [8, 8], [3, 0], [1, 1], [[1, 4, 8], []])
    w = wl.make_custom(pr, 1, 1, 64, dtype=torch.float32, seed=3)
    lg = np.array([[1.5, 1.5], [0.25, 0.25], [0.0, 1e-30]], np.float32)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    got = ver.first_reject(torch.from_numpy(lg).to(ver.device), 0.0, 0).cpu().numpy()
    exp = orc.first_reject(lg, pr.num_segments, pr.boundaries, 0.0, 0)
    assert np.array_equal(got, exp)
    assert got[1].tolist() == [0, -1, 0, 0]


def _work_list(ver):
    """The tile work list as the attention kernel reads it, parsed from the plan blob (header of 32
    ints: n_q_tiles at 4, tile_m at 5, tile_n at 6, off_tiles at 24, off_work at 25)."""
    blob = ver.plan.view(torch.int32).cpu().numpy()
    n, off_tiles, off_work = int(blob[4]), int(blob[24]), int(blob[25])
    assert blob[5] == 32 and blob[6] == 64
    tiles = blob[off_tiles:off_tiles + 8 * n].reshape(n, 8)
    work = blob[off_work:off_work + 8 * n].reshape(n, 8)
    return tiles, work


def check_tiles_of_request(tiles, t, tok_base_want, M):
    """Tile classifier of one request against its dense mask M (oracle): every visible (row, key)
    pair lies in a listed key tile, tiles listed as fully visible are, listed tiles hold a visible
    pair.  `t` is the index of the request's first tile; returns the index after its last."""
    n = M.shape[0]
    nkt = (n + 63) // 64
    Mp = np.zeros((n, nkt * 64), dtype=np.uint8)
    Mp[:, :n] = M
    for t0 in range(0, n, 32):
        tok_base, tt0, rows, n_full, n_a, jb0, jb1, _ = (int(x) for x in tiles[t])
        assert (tok_base, tt0, rows) == (tok_base_want, t0, min(32, n - t0))
        blk = Mp[t0:t0 + rows].reshape(rows, nkt, 64)
        any_vis = blk.any(axis=(0, 2))
        all_vis = blk.all(axis=(0, 2))
        listed = np.zeros(nkt, dtype=bool)
        listed[:n_a] = True
        listed[jb0:jb1] = True
        assert 0 <= n_full <= n_a <= jb0 <= jb1 <= nkt
        assert not (any_vis & ~listed).any(), t0                 # nothing visible is skipped
        assert all_vis[:n_full].all(), t0                        # unmasked tiles really are
        # the classifier is tight: listed tiles hold a visible pair
        assert any_vis[listed].all(), t0
        t += 1
    return t


def check_work_order(tiles, work):
    cost = tiles[:, 4] + (tiles[:, 6] - tiles[:, 5])
    order = np.argsort(-cost, kind="stable")
    assert np.array_equal(work, tiles[order])


def check_work_list(pr):
    """Tile classifier against the oracle's dense mask, and the work list = the tile list sorted
    longest first (stable)."""
    w = wl.make_custom(pr, 4, 2, 64, dtype=torch.float32, seed=1)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    torch.cuda.synchronize()
    tiles, work = _work_list(ver)
    cu = pr.token_offsets()
    t = 0
    for b in range(pr.batch):
        M = orc.dense_mask(pr.prompt_len[b], pr.draft_len[b], pr.segment_len[b], pr.boundaries[b])
        t = check_tiles_of_request(tiles, t, cu[b], M)
    assert t == len(tiles)
    check_work_order(tiles, work)


@pytest.mark.parametrize("idx", range(len(EDGE_PROBLEMS)))
def test_work_list_edge_cases(idx):
    check_work_list(EDGE_PROBLEMS[idx])


def test_work_list_8b_single_launch_plan():
    check_work_list(wl.make("8b").problem)


def test_work_list_multi_kernel_plan():
    # more than 8192 tokens: the plan is built by the separate upload / tokens / tiles / ranking
    # kernels instead of the single-workgroup kernel
    rng = np.random.default_rng(11)
    B = 6
    P = [int(x) for x in rng.integers(0, 700, B)]
    T = [int(x) for x in rng.integers(3000, 6000, B)]
    K = [int(x) for x in rng.integers(0, 9, B)]
    S = [int(x) for x in rng.integers(1, 70, B)]
    bounds = [sorted(int(x) for x in rng.integers(0, T[b] + 1, K[b])) for b in range(B)]
    pr = wl.Problem(P, T, K, S, bounds)
    assert pr.total_tokens > 8192
    check_work_list(pr)


def test_binding_refuses_host_and_strided_tensors():
    # the binding passes raw addresses to kernels: anything that is not contiguous memory of the
    # current GPU must be stopped in Python, before a launch
    w = wl.make("tiny")
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    out = torch.empty_like(q)
    with pytest.raises(ValueError):
        ver.attention(w.q, k, v, out=out)                                   # q in host memory
    with pytest.raises(ValueError):
        ver.attention(q, k, v, out=torch.empty(q.shape, dtype=q.dtype))     # out in host memory
    wide = torch.empty(q.shape[0], q.shape[1], 2 * q.shape[2], dtype=q.dtype, device=dev)
    with pytest.raises(ValueError):
        ver.attention(q, k, v, out=wide[:, :, :q.shape[2]])                 # strided view
    with pytest.raises(ValueError):
        ver.first_reject(torch.zeros(ver.sizes.total_segments, 2), 0.0)     # logits in host memory
    torch.cuda.synchronize()


def _random_problem(rng):
    B = int(rng.integers(1, 5))
    P = [int(x) for x in rng.integers(0, 150, B)]
    T = [int(x) for x in rng.integers(1, 400, B)]
    K = [int(x) for x in rng.integers(0, 9, B)]
    S = [int(rng.choice([1, 2, 5, 16, 31, 32, 33, 64, 70])) for _ in range(B)]
    bounds = [sorted(int(x) for x in rng.integers(0, T[b] + 1, K[b])) for b in range(B)]
    return wl.Problem(P, T, K, S, bounds)


@pytest.mark.parametrize("seed", range(12))
def test_random_plans_both_layouts(seed):
    # seeded random structures (ragged batches, repeated and zero boundaries, segments shorter and longer
    # than a tile), ten per case: dense mask, positions and judge rows bit-exact in both packings, the
    # tile work list against the oracle's mask, and the readout
    import dataclasses
    rng = np.random.default_rng(9100 + seed)
    for _ in range(10):
        pr = _random_problem(rng)
        check_plan(pr)
        check_work_list(pr)
        pri = dataclasses.replace(pr, layout=1)
        w = wl.make_custom(pri, 4, 2, 64, dtype=torch.float32, seed=1)
        ver = gc.make_verifier(pv, w, dense_mask=True)
        ver.build_mask()
        pos, ae, bs, jr = pv.pv_plan_export(ver.sizes, ver.plan)
        torch.cuda.synchronize()
        assert np.array_equal(ver.dense_mask.cpu().numpy(), gc.oracle_dense_mask_flat(pri))
        opos, ojr = gc.oracle_plan_arrays(pri)
        assert np.array_equal(pos.cpu().numpy().astype(np.int64), opos)
        assert np.array_equal(jr.cpu().numpy().astype(np.int64), ojr)
        thr = orc.margin_threshold(0.9)
        for mode in (0, 1):
            got = ver.first_reject(w.logits.cuda(), thr, mode).cpu().numpy()
            assert np.array_equal(got, orc.first_reject(w.logits.numpy(), pr.num_segments, pr.boundaries, thr, mode))


def check_quad_list(pr):
    """Groups of four consecutive query tiles (the work items of group sizes other than 4 and 8): every
    group of every request appears once, last group of a request first, and its key-tile list holds every
    key tile that any of its rows can see."""
    w = wl.make_custom(pr, 5, 1, 64, dtype=torch.float32, seed=1)
    ver = gc.make_verifier(pv, w)
    ver.build_mask()
    torch.cuda.synchronize()
    blob = ver.plan.view(torch.int32).cpu().numpy()
    n_quads, off_quadwork = int(blob[33]), int(blob[35])        # header ints 33..35: n_quads, off_quad_start, off_quadwork
    assert n_quads == ver.sizes.n_quads == sum(((pr.seq_len(b) + 31) // 32 + 3) // 4 for b in range(pr.batch))
    quads = blob[off_quadwork:off_quadwork + 8 * n_quads].reshape(n_quads, 8)
    tiles, _ = _work_list(ver)
    cu = pr.token_offsets()
    at = 0
    tile0 = 0
    for b in range(pr.batch):
        n = pr.seq_len(b)
        M = orc.dense_mask(pr.prompt_len[b], pr.draft_len[b], pr.segment_len[b], pr.boundaries[b])
        nkt = (n + 63) // 64
        Mp = np.zeros((n, nkt * 64), dtype=np.uint8)
        Mp[:, :n] = M
        n_tiles = (n + 31) // 32
        nq = (n_tiles + 3) // 4
        for pos in range(nq):
            ql = nq - 1 - pos                                   # last group first
            tok_base, t0, rows, first_tile, n_a, jb0, jb1, _ = (int(x) for x in quads[at + pos])
            assert (tok_base, t0, rows) == (cu[b], 128 * ql, min(128, n - 128 * ql))
            assert first_tile == tile0 + 4 * ql and int(tiles[first_tile][1]) == t0
            any_vis = Mp[t0:t0 + rows].reshape(rows, nkt, 64).any(axis=(0, 2))
            listed = np.zeros(nkt, dtype=bool)
            listed[:n_a] = True
            listed[jb0:jb1] = True
            assert 0 <= n_a <= jb0 <= jb1 <= nkt
            assert not (any_vis & ~listed).any(), (b, ql)
        at += nq
        tile0 += n_tiles


@pytest.mark.parametrize("idx", range(len(EDGE_PROBLEMS)))
def test_quad_list_edge_cases(idx):
    check_quad_list(EDGE_PROBLEMS[idx])


def test_quad_list_random_and_named():
    rng = np.random.default_rng(77)
    for _ in range(25):
        check_quad_list(_random_problem(rng))
    check_quad_list(wl.make("14b").problem)
    # more than 8192 tokens: the plan is built by the separate kernels, not by the single-workgroup one
    check_quad_list(wl.Problem([100, 7], [9000, 300], [3, 2], [40, 5], [[10, 4000, 9000], [0, 300]]))
