"""Seeded synthetic workloads for parallel prefix verification.

This module only draws shapes, boundaries and random tensors.  It holds none
of the method's arithmetic (no mask rule, no positions, no rotary embedding,
no softmax, no verdict rule): both the CPU oracle's tests and the HIP path's
tests/bench take their inputs from here so that the two see the same bits.

The paper measures end to end on public benchmarks with real models; none of
that is available or needed for the attention path, which consumes only
shapes and tensors.  The five named workloads below are synthetic stand-ins
with the structure of a packed verification pass (Section "Parallel Prefix
Verification"): a prompt, a draft of T tokens, and K suffix copies ("segments")
of S tokens, segment k being allowed to see the first p_k draft tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch


@dataclass
class Problem:
    """Structure of one packed batch (host side, plain integers)."""
    prompt_len: List[int]
    draft_len: List[int]
    num_segments: List[int]
    segment_len: List[int]
    boundaries: List[List[int]]          # per request, non-decreasing, 0 <= p <= T
    layout: int = 0                      # 0: segments appended after the draft; 1: each segment right after its chunk

    @property
    def batch(self) -> int:
        return len(self.prompt_len)

    def seq_len(self, b: int) -> int:
        return self.prompt_len[b] + self.draft_len[b] + self.num_segments[b] * self.segment_len[b]

    @property
    def total_tokens(self) -> int:
        return sum(self.seq_len(b) for b in range(self.batch))

    @property
    def total_segments(self) -> int:
        return sum(self.num_segments)

    def token_offsets(self) -> List[int]:
        cu = [0]
        for b in range(self.batch):
            cu.append(cu[-1] + self.seq_len(b))
        return cu

    def segment_offsets(self) -> List[int]:
        cu = [0]
        for b in range(self.batch):
            cu.append(cu[-1] + self.num_segments[b])
        return cu

    def flat_boundaries(self) -> List[int]:
        return [p for bs in self.boundaries for p in bs]


@dataclass
class Workload:
    name: str
    problem: Problem
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: torch.dtype                   # dtype of q/k/v handed to both sides
    rope_theta: float                    # 0 => no rotary embedding
    q: torch.Tensor                      # [total_tokens, Hq, D]
    k: torch.Tensor                      # [total_tokens, Hkv, D]
    v: torch.Tensor                      # [total_tokens, Hkv, D]
    logits: torch.Tensor                 # [total_segments, 2] fp32 = (l_correct, l_incorrect)
    tau: float                           # judge confidence threshold for the readout
    seed: int
    notes: dict = field(default_factory=dict)


def _sorted_distinct_uniform(rng: np.random.Generator, lo: int, hi: int, count: int) -> List[int]:
    """`count` distinct integers drawn uniformly from [lo, hi], sorted."""
    span = hi - lo + 1
    if count > span:
        raise ValueError("not enough distinct positions")
    picks = rng.choice(span, size=count, replace=False)
    return sorted(int(lo + x) for x in picks)


def _randn(gen: torch.Generator, *shape) -> torch.Tensor:
    return torch.randn(*shape, generator=gen, dtype=torch.float32)


def _judge_logits(rng: np.random.Generator, problem: Problem) -> torch.Tensor:
    """Per-segment (l_correct, l_incorrect) pairs with the usual shape of a
    verification run: confident Correct verdicts up to a random first error,
    mostly Incorrect (noisy) afterwards."""
    rows = []
    for b in range(problem.batch):
        K = problem.num_segments[b]
        first_err = int(rng.integers(0, K + 1))
        for k in range(K):
            base = rng.normal(0.0, 2.0)
            margin = rng.normal(6.0, 1.5) if k < first_err else rng.normal(-3.0, 3.0)
            rows.append((base + 0.5 * margin, base - 0.5 * margin))
    if not rows:
        return torch.zeros(0, 2, dtype=torch.float32)
    return torch.tensor(np.asarray(rows, dtype=np.float32))


def _tensors(seed: int, n_tok: int, hq: int, hkv: int, d: int, dtype: torch.dtype, scale: float = 1.0):
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    q = (_randn(gen, n_tok, hq, d) * scale).to(dtype)
    k = (_randn(gen, n_tok, hkv, d) * scale).to(dtype)
    v = (_randn(gen, n_tok, hkv, d) * scale).to(dtype)
    return q, k, v


def make_custom(problem: Problem, n_q_heads: int, n_kv_heads: int, head_dim: int,
                dtype: torch.dtype = torch.bfloat16, rope_theta: float = 0.0, seed: int = 0,
                value_scale: float = 1.0, tau: float = 0.985, name: str = "custom") -> Workload:
    """Random N(0,1)*value_scale tensors for an arbitrary structure (edge-case tests)."""
    q, k, v = _tensors(seed, problem.total_tokens, n_q_heads, n_kv_heads, head_dim, dtype, value_scale)
    rng = np.random.default_rng(seed + 7)
    return Workload(name, problem, n_q_heads, n_kv_heads, head_dim, dtype, rope_theta,
                    q, k, v, _judge_logits(rng, problem), tau, seed)


def make_tiny(seed: int = 1000, rope_theta: float = 0.0) -> Workload:
    """1 head, D=64, fp32; prompt 32 + draft 256; 4 segments of 16 tokens; boundaries 4 sorted
    distinct uniform positions in [16, 256]; Q/K/V = N(0,1)/sqrt(64); judge logit N(0,1) against a
    fixed 0 for the Incorrect class with tau = 0.5, i.e. "reject if logit < 0"."""
    rng = np.random.default_rng(seed)
    P, T, K, S = 32, 256, 4, 16
    prob = Problem([P], [T], [K], [S], [_sorted_distinct_uniform(rng, 16, T, K)])
    q, k, v = _tensors(seed, prob.total_tokens, 1, 1, 64, torch.float32, 1.0 / 8.0)
    lc = torch.tensor(rng.normal(0.0, 1.0, size=K).astype(np.float32))
    logits = torch.stack([lc, torch.zeros_like(lc)], dim=1).contiguous()
    return Workload("tiny", prob, 1, 1, 64, torch.float32, rope_theta, q, k, v, logits, 0.5, seed)


def make_8b(seed: int = 2000) -> Workload:
    """32 q heads / 8 kv heads, D=128, bf16; prompt 512 + draft 2048; 16 segments of 32 tokens;
    boundaries at sentence-like gaps: cumulative max(1, Poisson(96)) clipped to the draft length."""
    rng = np.random.default_rng(seed)
    P, T, K, S = 512, 2048, 16, 32
    gaps = np.maximum(1, rng.poisson(96.0, size=K))
    bounds = [int(min(T, x)) for x in np.cumsum(gaps)]
    prob = Problem([P], [T], [K], [S], [bounds])
    q, k, v = _tensors(seed, prob.total_tokens, 32, 8, 128, torch.bfloat16)
    return Workload("8b", prob, 32, 8, 128, torch.bfloat16, 5e5, q, k, v,
                    _judge_logits(rng, prob), 0.985, seed)


def make_8b_full_verify(seed: int = 2500) -> Workload:
    """The full-answer verification of the 8B-like shape: the same heads, prompt 512 + draft 2048, and no
    segment at all (K = 0), i.e. one plain causal pass whose single judgment is read at the last token."""
    prob = Problem([512], [2048], [0], [1], [[]])
    q, k, v = _tensors(seed, prob.total_tokens, 32, 8, 128, torch.bfloat16)
    return Workload("8b_full_verify", prob, 32, 8, 128, torch.bfloat16, 5e5, q, k, v,
                    torch.zeros(0, 2, dtype=torch.float32), 0.998, seed)


def make_ragged(seed: int = 3000, batch: int = 16) -> Workload:
    """8B-like heads, bf16; `batch` requests with prompt U[128,1024], draft U[512,4096],
    K U[4,32] segments of 32 tokens; boundaries K distinct sorted uniform on [16, T]."""
    rng = np.random.default_rng(seed)
    Ps, Ts, Ks, Ss, Bs = [], [], [], [], []
    for _ in range(batch):
        P = int(rng.integers(128, 1025))
        T = int(rng.integers(512, 4097))
        K = int(rng.integers(4, 33))
        Ps.append(P); Ts.append(T); Ks.append(K); Ss.append(32)
        Bs.append(_sorted_distinct_uniform(rng, 16, T, K))
    prob = Problem(Ps, Ts, Ks, Ss, Bs)
    q, k, v = _tensors(seed, prob.total_tokens, 32, 8, 128, torch.bfloat16)
    return Workload("ragged", prob, 32, 8, 128, torch.bfloat16, 5e5, q, k, v,
                    _judge_logits(rng, prob), 0.985, seed)


def make_14b(seed: int = 4000) -> Workload:
    """40 q heads / 8 kv heads (group of 5), D=128, bf16; prompt 1024 + draft 4096; 32 segments of
    48 tokens; boundary k at min(T, 128(k+1) + U{-32..32}); K has heavy-tailed outlier channels:
    4 seeded channels per kv head are 4 x Student-t(df=3) instead of N(0,1).  No rotary embedding."""
    rng = np.random.default_rng(seed)
    P, T, K, S = 1024, 4096, 32, 48
    bounds = [int(min(T, 128 * (i + 1) + rng.integers(-32, 33))) for i in range(K)]
    prob = Problem([P], [T], [K], [S], [bounds])
    hq, hkv, d = 40, 8, 128
    q, k, v = _tensors(seed, prob.total_tokens, hq, hkv, d, torch.float32)
    channels = {}
    for h in range(hkv):
        ch = sorted(int(c) for c in rng.choice(d, size=4, replace=False))
        channels[h] = ch
        t = rng.standard_t(3.0, size=(prob.total_tokens, 4)).astype(np.float32) * 4.0
        k[:, h, ch] = torch.from_numpy(t)
    bf = torch.bfloat16
    return Workload("14b", prob, hq, hkv, d, bf, 0.0, q.to(bf), k.to(bf), v.to(bf),
                    _judge_logits(rng, prob), 0.985, seed, {"outlier_channels": channels})


def make_70b(seed: int = 5000, batch: int = 4) -> Workload:
    """64 q heads / 8 kv heads, D=128, bf16; batch 4 of prompt 2048 + draft 8192; 64 segments of 64
    tokens; boundaries 64 distinct sorted uniform on [16, T] per request."""
    rng = np.random.default_rng(seed)
    P, T, K, S = 2048, 8192, 64, 64
    prob = Problem([P] * batch, [T] * batch, [K] * batch, [S] * batch,
                   [_sorted_distinct_uniform(rng, 16, T, K) for _ in range(batch)])
    q, k, v = _tensors(seed, prob.total_tokens, 64, 8, 128, torch.bfloat16)
    return Workload("70b", prob, 64, 8, 128, torch.bfloat16, 5e5, q, k, v,
                    _judge_logits(rng, prob), 0.985, seed)


def quantize_fp8(x: torch.Tensor):
    """Storage conversion of a [tokens, heads, D] tensor to FP8 E4M3 codes with one scale per head
    (scale = largest magnitude of the head / 448, the largest E4M3 value; library rounding).
    Returns (codes uint8 [tokens, heads, D], scales float32 [heads])."""
    xf = x.float()
    scale = (xf.abs().amax(dim=(0, 2)) / 448.0).clamp_min(2.0 ** -20)
    codes = (xf / scale[None, :, None]).to(torch.float8_e4m3fn).view(torch.uint8)
    return codes.contiguous(), scale.contiguous()


WORKLOADS = {
    "tiny": make_tiny,
    "8b": make_8b,
    "8b_full_verify": make_8b_full_verify,
    "ragged": make_ragged,
    "14b": make_14b,
    "70b": make_70b,
}


def make(name: str, seed: Optional[int] = None, **kw) -> Workload:
    fn = WORKLOADS[name]
    return fn(**kw) if seed is None else fn(seed=seed, **kw)
