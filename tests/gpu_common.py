"""Helpers shared by the GPU parity tests (run the HIP path through the C ABI binding and the
oracle on the same seeded inputs)."""
import numpy as np
import torch

import pv_workloads as wl
from oracle import pv_oracle as orc


def device():
    return torch.device("cuda:0")


def make_verifier(pv, w, dense_mask=False):
    pr = w.problem
    return pv.Verifier(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len,
                       pr.flat_boundaries(), w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype,
                       dense_mask=dense_mask, layout=pr.layout)


def run_gpu_attention(pv, w, out_dtype=None, lse=False, ver=None, softmax_scale=0.0):
    if ver is None:
        ver = make_verifier(pv, w)
        ver.build_mask()
    dev = ver.device
    q, k, v = w.q.to(dev), w.k.to(dev), w.v.to(dev)
    out = torch.empty(q.shape, dtype=out_dtype or w.dtype, device=dev)
    l = torch.empty(w.n_q_heads, w.problem.total_tokens, dtype=torch.float32, device=dev) if lse else None
    ver.attention(q, k, v, out=out, lse=l, rope_theta=w.rope_theta, softmax_scale=softmax_scale)
    torch.cuda.synchronize()
    return (out, l) if lse else out


def oracle_attention(w, rows_per_request=None, return_lse=False, scale=None):
    pr = w.problem
    return orc.masked_attention(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len,
                                pr.boundaries, w.q.double().numpy(), w.k.double().numpy(),
                                w.v.double().numpy(), rope_theta=w.rope_theta, scale=scale,
                                rows_per_request=rows_per_request, return_lse=return_lse, layout=pr.layout)


def oracle_dense_mask_flat(pr):
    parts = []
    mask_fn = orc.dense_mask_interleaved if pr.layout == orc.LAYOUT_INTERLEAVED else orc.dense_mask
    for b in range(pr.batch):
        parts.append(mask_fn(pr.prompt_len[b], pr.draft_len[b], pr.segment_len[b],
                             pr.boundaries[b]).reshape(-1))
    return np.concatenate(parts)


def oracle_plan_arrays(pr):
    pos, jr = [], []
    cu = pr.token_offsets()
    for b in range(pr.batch):
        P, T, K, S = pr.prompt_len[b], pr.draft_len[b], pr.num_segments[b], pr.segment_len[b]
        if pr.layout == orc.LAYOUT_INTERLEAVED:
            pos.append(orc.positions_interleaved(P, T, S, pr.boundaries[b]))
            jr.append(orc.judge_rows_interleaved(P, T, S, pr.boundaries[b]) + cu[b])
        else:
            pos.append(orc.positions(P, T, S, pr.boundaries[b]))
            jr.append(orc.judge_rows(P, T, S, K) + cu[b])
    return np.concatenate(pos), np.concatenate(jr) if jr else np.zeros(0, np.int64)


def sample_rows(pr, n_random=128, seed=0, max_multiples=24):
    """Per request: first/last two rows of the prompt, the draft and of up to four segments
    (first, last, two in the middle), rows next to multiples of 32/64/128, and seeded random rows."""
    rng = np.random.default_rng(seed)
    out = []
    for b in range(pr.batch):
        P, T, K, S = pr.prompt_len[b], pr.draft_len[b], pr.num_segments[b], pr.segment_len[b]
        N = pr.seq_len(b)
        rows = set()
        def ends(lo, hi):
            for r in (lo, lo + 1, hi - 2, hi - 1):
                if lo <= r < hi:
                    rows.add(r)
        ends(0, P)
        ends(P, P + T)
        for k in sorted(set([0, K // 3, (2 * K) // 3, K - 1])):
            if 0 <= k < K:
                ends(P + T + k * S, P + T + (k + 1) * S)
        mult = [m for step in (32, 64, 128) for m in range(step, N, step)]
        if len(mult) > max_multiples:
            mult = list(rng.choice(mult, size=max_multiples, replace=False))
        for m in mult:
            for r in (m - 1, m, m + 1):
                if 0 <= r < N:
                    rows.add(int(r))
        for r in rng.integers(0, N, size=n_random):
            rows.add(int(r))
        out.append(sorted(rows))
    return out


def packed_row_index(pr, rows_per_request):
    cu = pr.token_offsets()
    return np.concatenate([np.asarray(r, dtype=np.int64) + cu[b] for b, r in enumerate(rows_per_request)])
