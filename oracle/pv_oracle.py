"""CPU oracle for parallel prefix verification -- TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy.  Only tests, the smoke check and the benchmark's CPU
baseline may import this file; the product (the HIP library and its Python
binding) never does, and this file imports nothing from the product.

What it computes, and the passages it follows (paper section "Parallel Prefix
Verification", and appendix "Detailed Algorithm": "Notation and judge
calibration", "Parallel partial verify", "Adopted-prefix length"):

* `dense_mask`      the custom attention mask of the packed verification pass,
                    materialised entry by entry from the visibility rules of
                    "Parallel Prefix Verification".
* `positions`       rotary positions: prompt and draft count up from 0; suffix
                    copy k continues from the end of the prefix it judges, so
                    that its judgment position receives the same input as a
                    stand-alone run of that prefix followed by the suffix.
* `rope`            rotary embedding, half-split pairing.
* `attention`       softmax(mask(Q K^T * scale)) V for one request, no tiling.
* `*_interleaved`   the same pass in the packing of "Parallel partial verify": every suffix
                    copy (End slot) directly after its chunk instead of after the draft.
* `decode_e4m3`, `masked_attention_fp8kv`
                    the same pass with K and V stored as FP8 codes plus a scale per kv head
                    (the paper's target checkpoints are FP8; reading: see the function).
* `first_reject`    two-way confidence verdicts (Eq. for p_2w), the last-correct
                    index k* ("Parallel partial verify"), the adopted length L*
                    (Eq. "adopted", with rollback eta = 0 generalised to arbitrary
                    boundaries) and the main-text rule t* = max{t_i : Correct}.

Readings where the paper is silent are listed in the design notes of this
repository; every function below is pinned by tests that do not reuse its
own formula (brute force over stand-alone sequences with a library attention,
closed-form counts, exhaustive enumeration).

Conventions (0-indexed).  One request has P prompt tokens, T draft tokens and
K suffix copies ("segments") of S tokens each, laid out
[prompt | draft | segment_0 | ... | segment_{K-1}], N = P + T + K*S tokens.
`boundaries[k] = p_k` is the number of draft tokens segment k may see.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------- mask

def dense_mask(P: int, T: int, S: int, boundaries: Sequence[int],
               rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """M[r, j] = 1 iff query token rows[r] may attend to key token j (uint8).

    Rules ("Parallel Prefix Verification"):
      * a prompt or draft token attends causally (to itself and everything before);
      * a token of suffix copy k attends to the whole prompt, to the draft tokens
        up through its boundary (the first p_k of them), causally to its own copy,
        and to nothing else -- never to another copy, never to later draft tokens.
    """
    K = len(boundaries)
    N = P + T + K * S
    if rows is None:
        rows = range(N)
    j = np.arange(N)
    key_is_prompt = j < P
    key_is_draft = (j >= P) & (j < P + T)
    key_draft_index = j - P                      # meaningful where key_is_draft
    key_is_segment = j >= P + T
    key_segment = np.where(key_is_segment, (j - P - T) // max(S, 1), -1)
    key_offset = np.where(key_is_segment, (j - P - T) % max(S, 1), -1)

    M = np.zeros((len(rows), N), dtype=np.uint8)
    for r, i in enumerate(rows):
        if i < P + T:
            visible = j <= i
        else:
            k = (i - P - T) // S
            a = (i - P - T) % S
            sees_prompt = key_is_prompt
            sees_draft = key_is_draft & (key_draft_index < boundaries[k])
            sees_self = key_is_segment & (key_segment == k) & (key_offset <= a)
            visible = sees_prompt | sees_draft | sees_self
        M[r] = visible
    return M


def positions(P: int, T: int, S: int, boundaries: Sequence[int]) -> np.ndarray:
    """Rotary position of every token (int64 [N])."""
    K = len(boundaries)
    pos = np.empty(P + T + K * S, dtype=np.int64)
    pos[:P + T] = np.arange(P + T)
    for k in range(K):
        start = P + T + k * S
        pos[start:start + S] = P + boundaries[k] + np.arange(S)
    return pos


def judge_rows(P: int, T: int, S: int, K: int) -> np.ndarray:
    """Row whose hidden state carries the verdict of segment k: its last token."""
    return np.array([P + T + (k + 1) * S - 1 for k in range(K)], dtype=np.int64)


# --------------------------------------------------------------------------- interleaved packing

LAYOUT_APPENDED, LAYOUT_INTERLEAVED = 0, 1


def interleaved_tokens(P: int, T: int, S: int, boundaries: Sequence[int]):
    """The packed prompt of "Parallel partial verify", token by token:
    prefix | C_1 | End_1 | C_2 | End_2 | ... | C_K | End_K | (draft tokens after the last boundary),
    where chunk C_k holds the draft tokens between boundary k-1 and boundary k and End_k is the
    k-th copy of the S-token judge suffix.  Returns a list of tuples
      ('q', i)        prefix token i,
      ('c', k, t)     draft token t, a member of chunk k (k = K for the tail after the last End),
      ('e', k, a)     token a of End slot k."""
    toks = [('q', i) for i in range(P)]
    prev = 0
    for k, p in enumerate(boundaries):
        toks += [('c', k, t) for t in range(prev, p)]
        toks += [('e', k, a) for a in range(S)]
        prev = p
    toks += [('c', len(boundaries), t) for t in range(prev, T)]
    return toks


def dense_mask_interleaved(P: int, T: int, S: int, boundaries: Sequence[int],
                           rows: Optional[Sequence[int]] = None) -> np.ndarray:
    """The mask of the interleaved packing ("Parallel partial verify"): an End slot attends to the
    question prefix, to its own prefix C_1..C_k, causally to itself, and to nothing else (no other
    End slot, no later chunk).  Prefix and chunk tokens are the ordinary causal sequence
    prefix + draft: a chunk token attends to the prefix and to the draft tokens up to itself, and
    never to an End slot (End slots are insertions the draft must not see)."""
    toks = interleaved_tokens(P, T, S, boundaries)
    N = len(toks)
    if rows is None:
        rows = range(N)
    kind = np.array([t[0] for t in toks])
    index = np.array([t[1] for t in toks])           # chunk or slot number (prefix: token index)
    j = np.arange(N)
    key_prefix, key_chunk, key_end = kind == 'q', kind == 'c', kind == 'e'
    M = np.zeros((len(rows), N), dtype=np.uint8)
    for r, i in enumerate(rows):
        not_later = j <= i                           # nothing attends forward
        if kind[i] == 'e':
            k = index[i]
            visible = key_prefix | (key_chunk & (index <= k)) | (key_end & (index == k))
        else:                                        # prefix or chunk token: the plain causal sequence
            visible = key_prefix | key_chunk
        M[r] = visible & not_later
    return M


def positions_interleaved(P: int, T: int, S: int, boundaries: Sequence[int]) -> np.ndarray:
    """Rotary positions in the interleaved packing: prefix and draft tokens keep the positions of
    the plain sequence prefix + draft; End slot k continues from the end of the prefix it judges."""
    pos = []
    for tok in interleaved_tokens(P, T, S, boundaries):
        if tok[0] == 'q':
            pos.append(tok[1])
        elif tok[0] == 'c':
            pos.append(P + tok[2])
        else:
            pos.append(P + boundaries[tok[1]] + tok[2])
    return np.asarray(pos, dtype=np.int64)


def judge_rows_interleaved(P: int, T: int, S: int, boundaries: Sequence[int]) -> np.ndarray:
    """Row of the last token of every End slot."""
    toks = interleaved_tokens(P, T, S, boundaries)
    where = {(t[1]): i for i, t in enumerate(toks) if t[0] == 'e' and t[2] == S - 1}
    return np.asarray([where[k] for k in range(len(boundaries))], dtype=np.int64)


# --------------------------------------------------------------------------- rotary

def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate x [N, H, D] (fp64) by angle pos * theta^(-2c/D) on the pair (c, c + D/2)."""
    if theta == 0.0:
        return x.copy()
    N, H, D = x.shape
    half = D // 2
    c = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * c / D)
    phi = pos.astype(np.float64)[:, None] * inv_freq[None, :]        # [N, half]
    cos = np.cos(phi)[:, None, :]
    sin = np.sin(phi)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * cos - hi * sin
    out[..., half:] = hi * cos + lo * sin
    return out


# --------------------------------------------------------------------------- attention

def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray,
              scale: Optional[float] = None, rows: Optional[Sequence[int]] = None,
              return_lse: bool = False):
    """Masked softmax attention of one request in fp64.

    q [N, Hq, D], k and v [N, Hkv, D] (already rotated), mask [len(rows), N] for the
    query rows `rows` (all rows if None).  Query head h uses kv head h // (Hq/Hkv).
    Returns O [len(rows), Hq, D] (and the natural-log normaliser [len(rows), Hq]).
    """
    N, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    if rows is None:
        rows = np.arange(N)
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), Hq, D), dtype=np.float64)
    lse = np.empty((len(rows), Hq), dtype=np.float64)
    allowed = mask.astype(bool)
    for h in range(Hq):
        g = h // G
        s = (q[rows, h, :] @ k[:, g, :].T) * scale                  # [R, N]
        s = np.where(allowed, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        denom = e.sum(axis=1, keepdims=True)
        out[:, h, :] = (e @ v[:, g, :]) / denom
        lse[:, h] = (m + np.log(denom))[:, 0]
    return (out, lse) if return_lse else out


def masked_attention(prompt_len, draft_len, num_segments, segment_len, boundaries,
                     q: np.ndarray, k: np.ndarray, v: np.ndarray, rope_theta: float = 0.0,
                     scale: Optional[float] = None, rows_per_request=None, return_lse: bool = False,
                     layout: int = LAYOUT_APPENDED):
    """The packed pass: every request of the batch, tokens concatenated request after request.

    `boundaries` is a list of per-request lists.  q/k/v hold the same values the GPU is
    given, widened to fp64.  `rows_per_request[b]` (optional) restricts request b to the
    listed local query rows; the outputs are then concatenated in that order.
    `layout` selects the packing of a request's tokens: suffix copies appended after the draft,
    or interleaved after their chunks ("Parallel partial verify").
    """
    mask_fn = dense_mask_interleaved if layout == LAYOUT_INTERLEAVED else dense_mask
    pos_fn = positions_interleaved if layout == LAYOUT_INTERLEAVED else positions
    outs, lses = [], []
    start = 0
    for b in range(len(prompt_len)):
        P, T, K, S = prompt_len[b], draft_len[b], num_segments[b], segment_len[b]
        N = P + T + K * S
        rows = None if rows_per_request is None else rows_per_request[b]
        pos = pos_fn(P, T, S, boundaries[b])
        qb = rope(np.asarray(q[start:start + N], dtype=np.float64), pos, rope_theta)
        kb = rope(np.asarray(k[start:start + N], dtype=np.float64), pos, rope_theta)
        vb = np.asarray(v[start:start + N], dtype=np.float64)
        M = mask_fn(P, T, S, boundaries[b], rows)
        o, l = attention(qb, kb, vb, M, scale, rows, return_lse=True)
        outs.append(o)
        lses.append(l)
        start += N
    O = np.concatenate(outs, axis=0)
    return (O, np.concatenate(lses, axis=0)) if return_lse else O


# --------------------------------------------------------------------------- FP8 keys and values

def decode_e4m3(bits: np.ndarray) -> np.ndarray:
    """Value of every 8-bit code of the OCP FP8 E4M3 format (1 sign, 4 exponent, 3 mantissa bits,
    bias 7, no infinities, S.1111.111 = NaN), exactly, as fp64.  The targets of the paper's
    experiments are FP8 checkpoints (Experiments, Setup); this is the storage format such a serving
    stack keeps K and V in."""
    b = np.asarray(bits, dtype=np.uint8).astype(np.int64)
    sign = np.where(b & 0x80, -1.0, 1.0)
    e = (b >> 3) & 0xF
    m = b & 0x7
    sub = (m / 8.0) * 2.0 ** -6                       # exponent field 0: no hidden one
    nor = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    val = sign * np.where(e == 0, sub, nor)
    return np.where((e == 15) & (m == 7), np.nan, val)


def masked_attention_fp8kv(prompt_len, draft_len, num_segments, segment_len, boundaries,
                           q: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray,
                           k_scale: np.ndarray, v_scale: np.ndarray, rope_theta: float = 0.0,
                           scale: Optional[float] = None, rows_per_request=None,
                           return_lse: bool = False, layout: int = LAYOUT_APPENDED):
    """The packed pass with K and V held as FP8 E4M3 codes and one fp32 scale per kv head:
    K[t, h, :] = decode(k_bits[t, h, :]) * k_scale[h], likewise V.  The keys are what a KV cache
    holds, i.e. already rotated at their positions when they were written: only Q is rotated here,
    at the plan's positions.  Everything else is `masked_attention`: the same mask, the same
    positions, untiled fp64 softmax.  q [tokens, Hq, D] holds the values the GPU is given, widened."""
    mask_fn = dense_mask_interleaved if layout == LAYOUT_INTERLEAVED else dense_mask
    pos_fn = positions_interleaved if layout == LAYOUT_INTERLEAVED else positions
    ks = np.asarray(k_scale, dtype=np.float32).astype(np.float64)[None, :, None]
    vs = np.asarray(v_scale, dtype=np.float32).astype(np.float64)[None, :, None]
    outs, lses = [], []
    start = 0
    for b in range(len(prompt_len)):
        P, T, K, S = prompt_len[b], draft_len[b], num_segments[b], segment_len[b]
        N = P + T + K * S
        rows = None if rows_per_request is None else rows_per_request[b]
        pos = pos_fn(P, T, S, boundaries[b])
        qb = rope(np.asarray(q[start:start + N], dtype=np.float64), pos, rope_theta)
        kb = decode_e4m3(k_bits[start:start + N]) * ks
        vb = decode_e4m3(v_bits[start:start + N]) * vs
        M = mask_fn(P, T, S, boundaries[b], rows)
        o, l = attention(qb, kb, vb, M, scale, rows, return_lse=True)
        outs.append(o)
        lses.append(l)
        start += N
    O = np.concatenate(outs, axis=0)
    return (O, np.concatenate(lses, axis=0)) if return_lse else O


# --------------------------------------------------------------------------- readout

def margin_threshold(tau: float) -> float:
    """Smallest logit margin l_C - l_I whose two-way confidence reaches tau."""
    return math.log(tau / (1.0 - tau))


def verdicts(logits: np.ndarray, threshold: float) -> np.ndarray:
    """Correct (True) iff the raw argmax is Correct (ties count as Correct) and the
    two-way confidence is at least tau, i.e. the fp64 margin reaches the threshold."""
    d = logits[:, 0].astype(np.float64) - logits[:, 1].astype(np.float64)
    return (d >= 0.0) & (d >= threshold)


def first_reject(logits: np.ndarray, num_segments: Sequence[int], boundaries, threshold: float,
                 mode: int = 0) -> np.ndarray:
    """Per request (first_reject, k_star, L_star, n_incorrect), int32 [B, 4].

    mode 0 ("Parallel partial verify"): k* is the largest k whose verdict is Correct with no
      Incorrect before it, so first_reject = k* + 1 is the first Incorrect index (K if none);
      L* is the boundary of chunk k* (0 when k* = -1, the restart case).
    mode 1 (main text): t* = max{t_i : prefix i is Correct}; k* is the index attaining it
      (the largest such index), first_reject is still the first Incorrect index.
    """
    out = np.zeros((len(num_segments), 4), dtype=np.int32)
    start = 0
    for b, K in enumerate(num_segments):
        ok = verdicts(logits[start:start + K], threshold)
        p = list(boundaries[b])
        first = K
        for kk in range(K):
            if not ok[kk]:
                first = kk
                break
        if mode == 0:
            k_star = first - 1
        else:
            k_star = -1
            for kk in range(K):
                if ok[kk]:
                    k_star = kk
        L_star = p[k_star] if k_star >= 0 else 0
        out[b] = (first, k_star, L_star, int(K - ok.sum()))
        start += K
    return out


# --------------------------------------------------------------------------- decision policy

LABEL_SM, LABEL_SM_LG, LABEL_LG = 0, 1, 2          # ship the draft / continue from L* / restart


def chunk_run_rules(ok: np.ndarray, rho: float, kappa: int):
    """The two reject rules of "Parallel partial verify" on a verdict sequence: the run of chunks
    rejects the draft when the fraction of Incorrect chunks exceeds rho, or when the trailing run of
    Incorrect chunks reaches kappa.  Returns (rejects, n_incorrect, trailing_incorrect)."""
    K = len(ok)
    n_inc = int(K - int(np.sum(ok)))
    trailing = 0
    for kk in range(K - 1, -1, -1):
        if ok[kk]:
            break
        trailing += 1
    frac_rule = K > 0 and float(n_inc) > float(rho) * float(K)
    run_rule = kappa > 0 and trailing >= kappa
    return bool(frac_rule or run_rule), n_inc, trailing


def adopted_prefix(k_star: int, eta: float, bounds: Sequence[int]) -> int:
    """Adopted-prefix length (the equation of that name): roll back eta chunks from the last correct
    boundary.  With chunk k ending at draft token bounds[k], Delta * floor(max(0, k* + 1 - eta))
    chunks kept means L* = bounds[m - 1] with m = floor(max(0, k* + 1 - eta)), and 0 for m = 0."""
    m = int(math.floor(max(0.0, float(k_star) + 1.0 - float(eta))))
    return int(bounds[m - 1]) if m >= 1 else 0


def decide(logits: np.ndarray, full_logits, num_segments: Sequence[int], boundaries, *,
           margin_chunk: float, margin_chunk_relaxed: float, margin_full: float,
           margin_full_relaxed: float, margin_short: Sequence[float], rho: float, kappa: int,
           eta: float, relaxed_count_min: int = 3, premature: bool = False) -> np.ndarray:
    """Per request the decision of the detailed algorithm after the judge logits are known.

    premature = False: Stages 2-6.  Stage 2 accepts when the full-answer verdict is Correct at
      the strict threshold; Stage 3 accepts drafts of at most len(margin_short) chunks whose
      full-answer confidence reaches the short-draft threshold of that chunk count
      (margin_short[K-1], already combined with the relaxed full threshold by the caller);
      Stage 5 accepts when the full-answer confidence reaches the relaxed threshold and every
      chunk's confidence reaches the relaxed chunk threshold; Stage 6 continues from L* > 0 or
      restarts.  All confidences are compared as fp64 logit margins.
    premature = True: the premature-PV early exit: abort drafting when the chunk rules reject (with
      the rho passed) or at least relaxed_count_min chunks are below the relaxed chunk threshold.

    Returns int32 [B, 12]: label (premature without abort: -1), deciding stage (2, 3, 5, 6;
    premature: 1 abort / 0 go on), L*,
    k*, first_reject, n_incorrect, trailing_incorrect, chunk_rules_reject, n_below_relaxed,
    full verdict (premature: -1), index of the least confident chunk (-1 if K = 0), K.
    """
    B = len(num_segments)
    out = np.zeros((B, 12), dtype=np.int32)
    start = 0
    for b, K in enumerate(num_segments):
        lg = logits[start:start + K]
        d = lg[:, 0].astype(np.float64) - lg[:, 1].astype(np.float64)
        ok = (d >= 0.0) & (d >= margin_chunk)
        first = K
        for kk in range(K):
            if not ok[kk]:
                first = kk
                break
        k_star = first - 1
        rejects, n_inc, trailing = chunk_run_rules(ok, rho, kappa)
        n_below = int(np.sum(d < margin_chunk_relaxed))
        argmin = int(np.argmin(d)) if K > 0 else -1       # first index of the minimum
        L_star = adopted_prefix(k_star, eta, boundaries[b])
        if premature:
            abort = rejects or n_below >= relaxed_count_min
            label = (LABEL_SM_LG if L_star > 0 else LABEL_LG) if abort else -1   # -1: keep drafting
            out[b] = (label, 1 if abort else 0, L_star, k_star, first, n_inc, trailing, int(rejects),
                      n_below, -1, argmin, K)
        else:
            dF = float(np.float64(full_logits[b][0]) - np.float64(full_logits[b][1]))
            vF = dF >= 0.0 and dF >= margin_full
            if vF:
                label, stage = LABEL_SM, 2
            elif 1 <= K <= len(margin_short) and dF >= margin_short[K - 1]:
                label, stage = LABEL_SM, 3
            elif dF >= margin_full_relaxed and n_below == 0:
                label, stage = LABEL_SM, 5
            else:
                label, stage = (LABEL_SM_LG if L_star > 0 else LABEL_LG), 6
            out[b] = (label, stage, L_star, k_star, first, n_inc, trailing, int(rejects), n_below,
                      int(vF), argmin, K)
        start += K
    return out


def short_draft_margins(tau_sd: float, tau_full_relaxed: float, max_chunks: int):
    """Short-draft thresholds of Stage 3 as margins: tau(K) = min(tau_sd + 0.02 (K - 1),
    tau_full_relaxed) for K = 1 .. max_chunks."""
    return [margin_threshold(min(tau_sd + 0.02 * (K - 1), tau_full_relaxed))
            for K in range(1, max_chunks + 1)]


def judge_logits(hidden: np.ndarray, w2: np.ndarray, rows: np.ndarray) -> np.ndarray:
    """(l_C, l_I) of every judged position: the hidden state at that row times the two lm-head
    rows of the Correct and Incorrect tokens, in fp64.  hidden [tokens, H], w2 [2, H]."""
    h = hidden[np.asarray(rows, dtype=np.int64)].astype(np.float64)
    return h @ w2.astype(np.float64).T
