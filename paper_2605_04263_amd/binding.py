"""Thin ctypes binding of libpv.so (see include/pv.h).

Argument marshalling only: torch tensors supply device memory and the current stream; every
step of the path runs in the library's HIP kernels.  There is no CPU fallback: if the shared
library is missing, importing this module fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PV_LIBRARY", os.path.join(_HERE, "libpv.so"))   # override: a developer build

PV_OK = 0
PV_ERR_NULL, PV_ERR_SHAPE, PV_ERR_BOUNDARY, PV_ERR_WORKSPACE = -1, -2, -3, -4
PV_ERR_ALIGN, PV_ERR_DTYPE, PV_ERR_ARCH, PV_ERR_HIP = -5, -6, -7, -8
PV_BF16, PV_F32 = 0, 1
PV_LAYOUT_APPENDED, PV_LAYOUT_INTERLEAVED = 0, 1


class PvProblem(C.Structure):
    _fields_ = [("batch", C.c_int32),
                ("prompt_len", C.POINTER(C.c_int32)),
                ("draft_len", C.POINTER(C.c_int32)),
                ("num_segments", C.POINTER(C.c_int32)),
                ("segment_len", C.POINTER(C.c_int32)),
                ("boundaries", C.POINTER(C.c_int32)),
                ("layout", C.c_int32)]


class PvSizes(C.Structure):
    _fields_ = [("batch", C.c_int64), ("total_tokens", C.c_int64), ("total_segments", C.c_int64),
                ("max_seq_len", C.c_int64), ("n_q_tiles", C.c_int64), ("padded_keys", C.c_int64),
                ("plan_bytes", C.c_int64), ("dense_mask_bytes", C.c_int64),
                ("attn_workspace_bytes", C.c_int64),
                ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("in_dtype", C.c_int32), ("tile_m", C.c_int32), ("tile_n", C.c_int32),
                ("n_short_rows", C.c_int32), ("layout", C.c_int32),
                ("n_seg_tiles", C.c_int32), ("n_quads", C.c_int32), ("n_short_seg_rows", C.c_int32)]


PV_MAX_SHORT_CHUNKS = 8
PV_LABEL_SM, PV_LABEL_SM_LG, PV_LABEL_LG = 0, 1, 2


class PvPolicy(C.Structure):
    _fields_ = [("margin_chunk", C.c_double), ("margin_chunk_relaxed", C.c_double),
                ("margin_full", C.c_double), ("margin_full_relaxed", C.c_double),
                ("margin_short", C.c_double * PV_MAX_SHORT_CHUNKS),
                ("rho", C.c_double), ("eta", C.c_double),
                ("kappa", C.c_int32), ("n_short", C.c_int32),
                ("relaxed_count_min", C.c_int32), ("premature", C.c_int32)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(LIB_PATH)
    P = C.POINTER
    lib.pv_query_sizes.argtypes = [P(PvProblem), C.c_int32, C.c_int32, C.c_int32, C.c_int32, P(PvSizes)]
    lib.pv_build_mask.argtypes = [P(PvProblem), P(PvSizes), C.c_void_p, C.c_int64, C.c_void_p,
                                  C.c_int64, C.c_void_p]
    lib.pv_masked_attention.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_float,
                                        C.c_void_p, C.c_int64, C.c_void_p]
    lib.pv_segment_attention.argtypes = lib.pv_masked_attention.argtypes
    lib.pv_masked_attention_fp8kv.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                              C.c_float, C.c_float, C.c_void_p, C.c_int64, C.c_void_p]
    lib.pv_prepare_kv.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_int64, C.c_int64, C.c_int64, C.c_float, C.c_void_p, C.c_int64, C.c_void_p]
    lib.pv_segment_attention_prepared.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                  C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p,
                                                  C.c_int32, C.c_float, C.c_float, C.c_void_p, C.c_int64,
                                                  C.c_void_p]
    lib.pv_prepared_workspace_bytes.argtypes = [P(PvSizes), C.c_int64, P(C.c_int64)]
    lib.pv_masked_attention_static.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_float,
                                               C.c_void_p]
    lib.pv_static_workspace_needed.argtypes = [P(PvSizes), P(C.c_int64)]
    lib.pv_first_reject.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_double, C.c_int32,
                                    C.c_void_p, C.c_void_p]
    lib.pv_plan_export.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_void_p]
    lib.pv_judge_logits.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.c_void_p, C.c_void_p]
    lib.pv_decide.argtypes = [P(PvSizes), C.c_void_p, C.c_void_p, C.c_void_p, P(PvPolicy),
                              C.c_void_p, C.c_void_p]
    lib.pv_margin_from_tau.argtypes = [C.c_double, P(C.c_double)]
    lib.pv_profile_enable.argtypes = [C.c_int32]
    lib.pv_profile_read.argtypes = [P(C.c_float)]
    lib.pv_profile_read_all.argtypes = [P(C.c_float), C.c_int32, P(C.c_int32)]
    for name in ("pv_query_sizes", "pv_build_mask", "pv_masked_attention", "pv_segment_attention", "pv_first_reject",
                 "pv_plan_export", "pv_profile_enable", "pv_profile_read", "pv_profile_read_all",
                 "pv_last_hip_error",
                 "pv_judge_logits", "pv_decide", "pv_margin_from_tau", "pv_masked_attention_static", "pv_prepare_kv", "pv_segment_attention_prepared",
                 "pv_prepared_workspace_bytes", "pv_masked_attention_fp8kv",
                 "pv_static_workspace_needed"):
        getattr(lib, name).restype = C.c_int32
    lib.pv_strerror.argtypes = [C.c_int32]
    lib.pv_strerror.restype = C.c_char_p
    lib.pv_version.restype = C.c_char_p
    return lib


lib = _load()


class PvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.pv_strerror(status).decode()
        if status == PV_ERR_HIP:
            msg += f" [hipError {lib.pv_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


def _check(status: int, where: str) -> None:
    if status != PV_OK:
        raise PvError(status, where)


def _i32(values: Sequence[int]):
    return (C.c_int32 * max(1, len(values)))(*values)


@dataclass
class HostProblem:
    """Keeps the ctypes arrays of a pv_problem alive."""
    struct: PvProblem
    keep: tuple


def make_problem(prompt_len: Sequence[int], draft_len: Sequence[int], num_segments: Sequence[int],
                 segment_len: Sequence[int], boundaries: Sequence[int],
                 layout: int = PV_LAYOUT_APPENDED) -> HostProblem:
    arrs = tuple(_i32(list(x)) for x in (prompt_len, draft_len, num_segments, segment_len, boundaries))
    s = PvProblem(len(prompt_len), *[C.cast(a, C.POINTER(C.c_int32)) for a in arrs], layout)
    return HostProblem(s, arrs)


def pv_query_sizes(problem: HostProblem, n_q_heads: int, n_kv_heads: int, head_dim: int,
                   in_dtype: int) -> PvSizes:
    out = PvSizes()
    _check(lib.pv_query_sizes(C.byref(problem.struct), n_q_heads, n_kv_heads, head_dim, in_dtype,
                              C.byref(out)), "pv_query_sizes")
    return out


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    # the library dereferences these on the GPU of the current stream: host memory or another
    # GPU's memory would fault there, so it is refused here
    if not t.is_cuda or t.device.index != torch.cuda.current_device():
        raise ValueError("tensor must live on the current GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def pv_build_mask(problem: HostProblem, sizes: PvSizes, plan: torch.Tensor,
                  dense_mask: Optional[torch.Tensor] = None) -> None:
    """Writes the plan (and optionally the uint8 dense mask) on the current stream."""
    _check(lib.pv_build_mask(C.byref(problem.struct), C.byref(sizes), _ptr(plan),
                             plan.numel() * plan.element_size(), _ptr(dense_mask),
                             0 if dense_mask is None else dense_mask.numel(), _stream()),
           "pv_build_mask")


def pv_masked_attention(sizes: PvSizes, plan: torch.Tensor, q: torch.Tensor, k: torch.Tensor,
                        v: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor,
                        lse: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                        rope_theta: float = 0.0, segments_only: bool = False) -> None:
    want = torch.float32 if sizes.in_dtype == PV_F32 else torch.bfloat16
    if q.dtype != want or k.dtype != want or v.dtype != want:
        raise ValueError("q/k/v dtype does not match sizes.in_dtype")
    n, hq, hkv, d = sizes.total_tokens, sizes.n_q_heads, sizes.n_kv_heads, sizes.head_dim
    if tuple(q.shape) != (n, hq, d) or tuple(k.shape) != (n, hkv, d) or tuple(v.shape) != (n, hkv, d) \
            or tuple(out.shape) != (n, hq, d):
        raise ValueError("q/k/v/out shapes do not match sizes")
    if lse is not None and (lse.dtype != torch.float32 or tuple(lse.shape) != (hq, n)):
        raise ValueError("lse must be float32 [Hq, total_tokens]")
    if out.dtype == torch.bfloat16:
        out_dtype = PV_BF16
    elif out.dtype == torch.float32:
        out_dtype = PV_F32
    else:
        raise ValueError("out must be bf16 or fp32")
    fn = lib.pv_segment_attention if segments_only else lib.pv_masked_attention
    _check(fn(C.byref(sizes), _ptr(plan), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), out_dtype,
              softmax_scale, rope_theta, _ptr(workspace), workspace.numel() * workspace.element_size(),
              _stream()),
           "pv_segment_attention" if segments_only else "pv_masked_attention")


def pv_masked_attention_fp8kv(sizes: PvSizes, plan: torch.Tensor, q: torch.Tensor, k_fp8: torch.Tensor,
                              v_fp8: torch.Tensor, k_scale: torch.Tensor, v_scale: torch.Tensor,
                              out: torch.Tensor, workspace: torch.Tensor, lse: Optional[torch.Tensor] = None,
                              softmax_scale: float = 0.0, rope_theta: float = 0.0) -> None:
    """K/V as E4M3 codes (uint8 [tokens, Hkv, 128]) with per-head scales (float32 [Hkv]); Q bf16."""
    n, hq, hkv, d = sizes.total_tokens, sizes.n_q_heads, sizes.n_kv_heads, sizes.head_dim
    if q.dtype != torch.bfloat16 or tuple(q.shape) != (n, hq, d) or tuple(out.shape) != (n, hq, d):
        raise ValueError("q must be bfloat16 [total_tokens, Hq, D], out the same shape")
    for t in (k_fp8, v_fp8):
        if t.dtype != torch.uint8 or tuple(t.shape) != (n, hkv, d):
            raise ValueError("k_fp8/v_fp8 must be uint8 [total_tokens, Hkv, D]")
    for t in (k_scale, v_scale):
        if t.dtype != torch.float32 or tuple(t.shape) != (hkv,):
            raise ValueError("k_scale/v_scale must be float32 [Hkv]")
    if lse is not None and (lse.dtype != torch.float32 or tuple(lse.shape) != (hq, n)):
        raise ValueError("lse must be float32 [Hq, total_tokens]")
    out_dtype = PV_F32 if out.dtype == torch.float32 else PV_BF16
    _check(lib.pv_masked_attention_fp8kv(C.byref(sizes), _ptr(plan), _ptr(q), _ptr(k_fp8), _ptr(v_fp8),
                                         _ptr(k_scale), _ptr(v_scale), _ptr(out), _ptr(lse), out_dtype,
                                         softmax_scale, rope_theta, _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream()),
           "pv_masked_attention_fp8kv")


def pv_prepare_kv(sizes: PvSizes, plan: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                  workspace: torch.Tensor, rope_theta: float = 0.0, first_token: int = 0,
                  last_token: Optional[int] = None, block_table: Optional[torch.Tensor] = None,
                  page_size: int = 0, key_capacity: int = 0) -> None:
    """Prepared keys of the tokens [first_token, last_token) into `workspace`.  k, v: dense
    [total_tokens, Hkv, D], or a page pool [n_pages, page_size, Hkv, D] with an int32 block table."""
    if k.dtype != torch.bfloat16 or v.dtype != torch.bfloat16:
        raise ValueError("k/v must be bfloat16")
    if block_table is not None and block_table.dtype != torch.int32:
        raise ValueError("block_table must be int32")
    last = sizes.total_tokens if last_token is None else last_token
    _check(lib.pv_prepare_kv(C.byref(sizes), _ptr(plan), _ptr(k), _ptr(v), _ptr(block_table), page_size,
                             first_token, last, key_capacity, rope_theta, _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _stream()), "pv_prepare_kv")


def pv_segment_attention_prepared(sizes: PvSizes, plan: torch.Tensor, q: torch.Tensor, k: torch.Tensor,
                                  v: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor,
                                  lse: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                                  rope_theta: float = 0.0, block_table: Optional[torch.Tensor] = None,
                                  page_size: int = 0, key_capacity: int = 0) -> None:
    """Segment rows against the keys pv_prepare_kv left in `workspace`."""
    out_dtype = PV_F32 if out.dtype == torch.float32 else PV_BF16
    _check(lib.pv_segment_attention_prepared(C.byref(sizes), _ptr(plan), _ptr(q), _ptr(k), _ptr(v),
                                             _ptr(block_table), page_size, key_capacity, _ptr(out), _ptr(lse),
                                             out_dtype,
                                             softmax_scale, rope_theta, _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream()),
           "pv_segment_attention_prepared")


def pv_prepared_workspace_bytes(sizes: PvSizes, key_capacity: int = 0) -> int:
    out = C.c_int64(0)
    _check(lib.pv_prepared_workspace_bytes(C.byref(sizes), key_capacity, C.byref(out)),
           "pv_prepared_workspace_bytes")
    return out.value


PV_STATIC_WORKSPACE_BYTES = 32 << 20


def pv_static_workspace_needed(sizes: PvSizes) -> int:
    out = C.c_int64(0)
    _check(lib.pv_static_workspace_needed(C.byref(sizes), C.byref(out)), "pv_static_workspace_needed")
    return out.value


def pv_masked_attention_static(sizes: PvSizes, plan: torch.Tensor, q: torch.Tensor, k: torch.Tensor,
                               v: torch.Tensor, out: torch.Tensor, lse: Optional[torch.Tensor] = None,
                               softmax_scale: float = 0.0, rope_theta: float = 0.0) -> None:
    """pv_masked_attention with the library's own fixed workspace (no workspace argument)."""
    out_dtype = PV_F32 if out.dtype == torch.float32 else PV_BF16
    _check(lib.pv_masked_attention_static(C.byref(sizes), _ptr(plan), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                          _ptr(lse), out_dtype, softmax_scale, rope_theta, _stream()),
           "pv_masked_attention_static")


def pv_segment_attention(sizes: PvSizes, plan: torch.Tensor, q: torch.Tensor, k: torch.Tensor,
                         v: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor,
                         lse: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                         rope_theta: float = 0.0) -> None:
    """Rows of the segments only; every other row of `out` / `lse` is left as it is."""
    pv_masked_attention(sizes, plan, q, k, v, out, workspace, lse, softmax_scale, rope_theta,
                        segments_only=True)


def pv_first_reject(sizes: PvSizes, plan: torch.Tensor, logits: torch.Tensor, margin_threshold: float,
                    mode: int, out: torch.Tensor) -> None:
    if logits.dtype != torch.float32 or tuple(logits.shape) != (sizes.total_segments, 2):
        raise ValueError("logits must be float32 [total_segments, 2]")
    if out.dtype != torch.int32 or tuple(out.shape) != (sizes.batch, 4):
        raise ValueError("out must be int32 [batch, 4]")
    _check(lib.pv_first_reject(C.byref(sizes), _ptr(plan), _ptr(logits) if logits.numel() else None,
                               margin_threshold, mode, _ptr(out), _stream()), "pv_first_reject")


def pv_judge_logits(sizes: PvSizes, plan: torch.Tensor, hidden: torch.Tensor, w2: torch.Tensor,
                    logits: torch.Tensor) -> None:
    if hidden.dtype != torch.bfloat16 or hidden.dim() != 2 or hidden.shape[0] != sizes.total_tokens:
        raise ValueError("hidden must be bfloat16 [total_tokens, hidden_size]")
    if w2.dtype != torch.bfloat16 or tuple(w2.shape) != (2, hidden.shape[1]):
        raise ValueError("w2 must be bfloat16 [2, hidden_size]")
    if logits.dtype != torch.float32 or tuple(logits.shape) != (sizes.total_segments, 2):
        raise ValueError("logits must be float32 [total_segments, 2]")
    if not (hidden.is_contiguous() and w2.is_contiguous() and logits.is_contiguous()):
        raise ValueError("tensors must be contiguous")
    _check(lib.pv_judge_logits(C.byref(sizes), _ptr(plan), _ptr(hidden), _ptr(w2), hidden.shape[1],
                               _ptr(logits) if logits.numel() else None, _stream()), "pv_judge_logits")


def make_policy(margin_chunk: float, margin_chunk_relaxed: float, margin_full: float,
                margin_full_relaxed: float, margin_short: Sequence[float], rho: float, kappa: int,
                eta: float, relaxed_count_min: int = 3, premature: bool = False) -> PvPolicy:
    if len(margin_short) > PV_MAX_SHORT_CHUNKS:
        raise ValueError("too many short-draft thresholds")
    pol = PvPolicy()
    pol.margin_chunk, pol.margin_chunk_relaxed = margin_chunk, margin_chunk_relaxed
    pol.margin_full, pol.margin_full_relaxed = margin_full, margin_full_relaxed
    for i, m in enumerate(margin_short):
        pol.margin_short[i] = m
    pol.rho, pol.eta, pol.kappa, pol.n_short = rho, eta, kappa, len(margin_short)
    pol.relaxed_count_min, pol.premature = relaxed_count_min, 1 if premature else 0
    return pol


def pv_decide(sizes: PvSizes, plan: torch.Tensor, logits: torch.Tensor,
              full_logits: Optional[torch.Tensor], policy: PvPolicy, out: torch.Tensor) -> None:
    if logits.dtype != torch.float32 or tuple(logits.shape) != (sizes.total_segments, 2):
        raise ValueError("logits must be float32 [total_segments, 2]")
    if full_logits is not None and (full_logits.dtype != torch.float32 or
                                    tuple(full_logits.shape) != (sizes.batch, 2)):
        raise ValueError("full_logits must be float32 [batch, 2]")
    if out.dtype != torch.int32 or tuple(out.shape) != (sizes.batch, 12):
        raise ValueError("out must be int32 [batch, 12]")
    _check(lib.pv_decide(C.byref(sizes), _ptr(plan), _ptr(logits) if logits.numel() else None,
                         _ptr(full_logits), C.byref(policy), _ptr(out), _stream()), "pv_decide")


def pv_plan_export(sizes: PvSizes, plan: torch.Tensor):
    """(positions, a_end, b_start, judge_row) as int32 device tensors."""
    dev = plan.device
    n, ns = sizes.total_tokens, sizes.total_segments
    pos, ae, bs = (torch.empty(n, dtype=torch.int32, device=dev) for _ in range(3))
    jr = torch.empty(max(ns, 1), dtype=torch.int32, device=dev)
    _check(lib.pv_plan_export(C.byref(sizes), _ptr(plan), _ptr(pos), _ptr(ae), _ptr(bs), _ptr(jr),
                              _stream()), "pv_plan_export")
    return pos, ae, bs, jr[:ns]


def pv_profile_enable(on: bool) -> None:
    _check(lib.pv_profile_enable(1 if on else 0), "pv_profile_enable")


def pv_profile_read() -> float:
    ms = C.c_float(0.0)
    _check(lib.pv_profile_read(C.byref(ms)), "pv_profile_read")
    return ms.value


PV_PROFILE_RING = 1024


def pv_profile_read_all() -> list:
    """Main-kernel durations (ms) of the attention calls since profiling was enabled, oldest first
    (the last PV_PROFILE_RING of them)."""
    buf = (C.c_float * PV_PROFILE_RING)()
    n = C.c_int32(0)
    _check(lib.pv_profile_read_all(buf, PV_PROFILE_RING, C.byref(n)), "pv_profile_read_all")
    return [buf[i] for i in range(n.value)]


def pv_margin_from_tau(tau: float) -> float:
    """The logit margin at which the two-way confidence equals tau (computed by the library)."""
    out = C.c_double(0.0)
    _check(lib.pv_margin_from_tau(tau, C.byref(out)), "pv_margin_from_tau")
    return out.value


margin_from_tau = pv_margin_from_tau


class Verifier:
    """Convenience holder of the device buffers of one problem (plan, workspace)."""

    def __init__(self, prompt_len, draft_len, num_segments, segment_len, boundaries_flat,
                 n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: torch.dtype,
                 device: str = "cuda:0", dense_mask: bool = False, layout: int = PV_LAYOUT_APPENDED):
        self.problem = make_problem(prompt_len, draft_len, num_segments, segment_len, boundaries_flat, layout)
        in_dtype = PV_F32 if dtype == torch.float32 else PV_BF16
        self.sizes = pv_query_sizes(self.problem, n_q_heads, n_kv_heads, head_dim, in_dtype)
        self.device = torch.device(device)
        self.plan = torch.empty(self.sizes.plan_bytes // 4, dtype=torch.int32, device=self.device)
        self.workspace = torch.empty(self.sizes.attn_workspace_bytes, dtype=torch.uint8, device=self.device)
        self.dense_mask = (torch.empty(self.sizes.dense_mask_bytes, dtype=torch.uint8, device=self.device)
                           if dense_mask else None)
        self.readout = torch.empty(self.sizes.batch, 4, dtype=torch.int32, device=self.device)

    def build_mask(self) -> None:
        pv_build_mask(self.problem, self.sizes, self.plan, self.dense_mask)

    def attention(self, q, k, v, out=None, lse=None, softmax_scale: float = 0.0, rope_theta: float = 0.0):
        if out is None:
            out = torch.empty_like(q)
        pv_masked_attention(self.sizes, self.plan, q, k, v, out, self.workspace, lse, softmax_scale, rope_theta)
        return out

    def segment_attention(self, q, k, v, out, lse=None, softmax_scale: float = 0.0, rope_theta: float = 0.0):
        pv_segment_attention(self.sizes, self.plan, q, k, v, out, self.workspace, lse, softmax_scale, rope_theta)
        return out

    def first_reject(self, logits, margin_threshold: float, mode: int = 0):
        pv_first_reject(self.sizes, self.plan, logits, margin_threshold, mode, self.readout)
        return self.readout

    def judge_logits(self, hidden, w2):
        logits = torch.empty(self.sizes.total_segments, 2, dtype=torch.float32, device=self.device)
        pv_judge_logits(self.sizes, self.plan, hidden, w2, logits)
        return logits

    def decide(self, logits, full_logits, policy: PvPolicy):
        out = torch.empty(self.sizes.batch, 12, dtype=torch.int32, device=self.device)
        pv_decide(self.sizes, self.plan, logits, full_logits, policy, out)
        return out
