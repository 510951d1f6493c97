"""Benchmark of the parallel-prefix-verification hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch already resident in HBM:
pv_build_mask -> pv_masked_attention (bf16 MFMA) -> pv_first_reject, one transformer layer.
Prints ONE JSON line.  `value` is effective (unmasked-pair) attention FLOPs per second of the
whole step; `roofline` prices the main attention kernel alone against the bf16 MFMA peak, its
duration measured with HIP events on the launch stream inside the timed steps; `cpu_baseline`
times the fp64 oracle on the host cores of the same box.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b|8b_full_verify|ragged|14b|70b|tiny]

A workload name with the suffix _fp8kv (8b_fp8kv, 70b_fp8kv, ...) is the same batch with K and V stored
as FP8 E4M3 codes and a scale per kv head, run through pv_masked_attention_fp8kv and priced against the
FP8 MFMA peak; the headline stays the bf16 `8b` workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
MFMA_FP8_PEAK_TFLOPS = 5000.0       # MI355X dense fp8 MFMA peak (workloads named *_fp8kv)



def measured_traffic_bytes(workload: str, kernel: str = "k_attn_bf16"):
    """HBM bytes per launch of the main kernel as measured under rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE, each scaled by what the same counter reads for a plain copy of known size): the
    figure is kept in the counter summary of the workload under profiles/, on a line
    `traffic_bytes_per_launch: <integer>`, next to the runs it came from.  None if there is no
    summary for this workload."""
    import re
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_counters.md")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*(\d+)", open(path).read(), flags=re.M)
    except OSError:
        return None
    return int(m.group(1)) if m else None


def unmasked_pairs(problem) -> int:
    """(query, key) pairs one head evaluates under the prefix mask."""
    total = 0
    for b in range(problem.batch):
        P, T, S = problem.prompt_len[b], problem.draft_len[b], problem.segment_len[b]
        c = P + T
        total += c * (c + 1) // 2
        for p in problem.boundaries[b]:
            total += S * (P + p) + S * (S + 1) // 2
    return total


def ensure_built() -> None:
    """Loads what is built; compiles only if there is no library or a source is newer than it."""
    from paper_2605_04263_amd import build
    if build.library_is_stale():
        build.build_library(verbose=False)


def cpu_baseline(w, eff_flops: float) -> dict:
    """The oracle as it stands, timed on this machine's host cores."""
    import numpy as np
    from oracle import pv_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    pr = w.problem
    q, k, v = w.q.double().numpy(), w.k.double().numpy(), w.v.double().numpy()
    full_pairs = unmasked_pairs(pr)
    # bounded sample: the whole workload if its dense fp64 work is small, else sampled rows
    dense = sum(pr.seq_len(b) ** 2 for b in range(pr.batch)) * w.n_q_heads * w.head_dim * 4
    if dense <= 4e11:
        rows, sample = None, "whole workload (every row, every head)"
        pairs = full_pairs
    else:
        rng = np.random.default_rng(0)
        budget = 2e11
        per_row = dense / pr.total_tokens
        n_rows = max(8, int(budget / per_row / pr.batch))
        rows = [sorted(set(int(x) for x in rng.integers(0, pr.seq_len(b), size=n_rows)))
                for b in range(pr.batch)]
        sample = f"{sum(len(r) for r in rows)} seeded random query rows (all heads) of {pr.total_tokens}"
        pairs = 0
        for b in range(pr.batch):
            mask_fn = orc.dense_mask_interleaved if pr.layout == orc.LAYOUT_INTERLEAVED else orc.dense_mask
            M = mask_fn(pr.prompt_len[b], pr.draft_len[b], pr.segment_len[b], pr.boundaries[b], rows[b])
            pairs += int(M.sum(dtype=np.int64))
    if w.name.endswith("_fp8kv"):
        import pv_workloads as wl
        kc, ksc = wl.quantize_fp8(w.k)
        vc, vsc = wl.quantize_fp8(w.v)
    t0 = time.perf_counter()
    if w.name.endswith("_fp8kv"):
        orc.masked_attention_fp8kv(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len, pr.boundaries,
                                   q, kc.numpy(), vc.numpy(), ksc.numpy(), vsc.numpy(), rope_theta=w.rope_theta,
                                   rows_per_request=rows, layout=pr.layout)
    else:
        orc.masked_attention(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len, pr.boundaries,
                             q, k, v, rope_theta=w.rope_theta, rows_per_request=rows, layout=pr.layout)
    orc.first_reject(w.logits.numpy(), pr.num_segments, pr.boundaries, orc.margin_threshold(w.tau), 0)
    dt = time.perf_counter() - t0
    flops = 4.0 * w.head_dim * w.n_q_heads * pairs
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": sample, "seconds": dt,
            "prefixes_per_s": pr.total_segments * (pairs / full_pairs) / dt}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step is ~0.1 ms: a few hundred warm-up steps let clocks and caches settle (20 are not enough:
    # the step then reads 4 % slower), and the timed loops still finish in a fraction of a second
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--settle-ms", type=float, default=300.0,
                    help="untimed steps run for this long before the warm-up so that the clocks of an idle "
                         "GPU have ramped up when the timed region starts (a step is ~0.1 ms: with a handful "
                         "of warm-up steps alone the main kernel reads 15-20 %% slower); 0 switches it off; "
                         "reported as settle_ms, steps and warmup stay as passed")
    ap.add_argument("--workload", default="8b")
    ap.add_argument("--layout", default="appended", choices=["appended", "interleaved"],
                    help="row order of the packed tensors: segments after the draft, or each after its chunk")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the untimed extra calls (decision calls, segment-only attention); used for "
                         "profiles so that every launch of the main kernel is one of the timed path")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    ensure_built()
    import torch
    import pv_workloads as wl
    from paper_2605_04263_amd import binding as pv

    if not torch.cuda.is_available():
        print("bench.py: needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    fp8kv = args.workload.endswith("_fp8kv")
    w = wl.make(args.workload[:-6] if fp8kv else args.workload)
    if fp8kv:
        import dataclasses
        w = dataclasses.replace(w, name=args.workload)
    pr = w.problem
    if args.layout == "interleaved":
        import dataclasses
        pr = dataclasses.replace(pr, layout=1)
        w = wl.Workload(**{**w.__dict__, "problem": pr})
    if w.dtype != torch.bfloat16:
        w = wl.make_custom(pr, w.n_q_heads, w.n_kv_heads, w.head_dim, torch.bfloat16, w.rope_theta, w.seed)
    ver = pv.Verifier(pr.prompt_len, pr.draft_len, pr.num_segments, pr.segment_len, pr.flat_boundaries(),
                      w.n_q_heads, w.n_kv_heads, w.head_dim, torch.bfloat16, layout=pr.layout)
    q, k, v, logits = w.q.to(dev), w.k.to(dev), w.v.to(dev), w.logits.to(dev)
    out = torch.empty_like(q)
    thr = pv.margin_from_tau(w.tau)
    if fp8kv:
        kc, ksc = (t.to(dev) for t in wl.quantize_fp8(w.k))
        vc, vsc = (t.to(dev) for t in wl.quantize_fp8(w.v))

        def attention():
            pv.pv_masked_attention_fp8kv(ver.sizes, ver.plan, q, kc, vc, ksc, vsc, out, ver.workspace,
                                         rope_theta=w.rope_theta)
    else:
        def attention():
            ver.attention(q, k, v, out=out, rope_theta=w.rope_theta)

    def step():
        ver.build_mask()
        attention()
        ver.first_reject(logits, thr, 0)

    pairs = unmasked_pairs(pr)
    eff_flops = 4.0 * w.head_dim * w.n_q_heads * pairs

    if args.calibrate_copy:       # a copy kernel of known size: 256 MiB read + 256 MiB written
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # settle phase: untimed, fixed wall time, reported
    settle_steps, t_settle = 0, time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(50):
            step()
        torch.cuda.synchronize()
        settle_steps += 50
    settle_ms = (time.perf_counter() - t_settle) * 1e3 if args.settle_ms > 0 else 0.0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # The same K steps once more, now with the library bracketing the main kernel of every
    # attention call with a pair of HIP events on the launch stream (recorded inside the loop,
    # never waited for there, read afterwards).  The event records themselves cost a few
    # microseconds per step, which is why `value` comes from the loop above.
    pv.pv_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t0) * 1e3 / args.steps
    ks = pv.pv_profile_read_all()          # one duration per step (the last PV_PROFILE_RING of them)
    pv.pv_profile_enable(False)
    kernel_ms = sum(ks) / len(ks)
    ks_sorted = sorted(ks)
    kernel_series = {"n": len(ks), "first": ks[0], "last": ks[-1], "min": ks_sorted[0],
                     "median": ks_sorted[len(ks) // 2], "p90": ks_sorted[min(len(ks) - 1, (9 * len(ks)) // 10)],
                     "max": ks_sorted[-1]}

    # per-call breakdown with events on the launch stream (untimed extra passes)
    def timed(fn, n=50):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / n
    n_b = max(5, min(50, args.steps))
    t_build = timed(ver.build_mask, n_b)
    t_attn = timed(attention, n_b)
    t_read = timed(lambda: ver.first_reject(logits, thr, 0), n_b)

    # the decision calls that follow the readout (not part of the timed step): lm-head gather of
    # the judge logits from hidden states of a 4096-wide model, and the full decision policy
    hid = torch.randn(pr.total_tokens, 4096, device=dev).bfloat16()
    w2 = (torch.randn(2, 4096, device=dev) * 0.05).bfloat16()
    full_lg = torch.zeros(pr.batch, 2, device=dev)
    pol = pv.make_policy(thr, pv.margin_from_tau(0.90), pv.margin_from_tau(0.998), pv.margin_from_tau(0.95),
                         [pv.margin_from_tau(0.95)] * 2, 0.30, 2, 0.0)
    # the same attention for the segment rows only (prompt and draft rows already evaluated by an
    # earlier pass): key pieces in parallel plus a merge
    seg_pairs = sum(pr.segment_len[b] * (pr.prompt_len[b] + p) + pr.segment_len[b] * (pr.segment_len[b] + 1) // 2
                    for b in range(pr.batch) for p in pr.boundaries[b])
    t_seg = t_seg_prepared = t_prepare = t_judge = t_decide = None
    if fp8kv:
        args.no_extras = True
    if not args.no_extras:
        if pr.total_segments:
            t_seg = timed(lambda: ver.segment_attention(q, k, v, out, rope_theta=w.rope_theta), n_b)
            # the same rows over keys prepared once (a second judge pass over the same prefix)
            t_prepare = timed(lambda: pv.pv_prepare_kv(ver.sizes, ver.plan, k, v, ver.workspace,
                                                       rope_theta=w.rope_theta), n_b)
            t_seg_prepared = timed(lambda: pv.pv_segment_attention_prepared(
                ver.sizes, ver.plan, q, k, v, out, ver.workspace, rope_theta=w.rope_theta), n_b)
        t_judge = timed(lambda: ver.judge_logits(hid, w2), n_b)
        t_decide = timed(lambda: ver.decide(logits, full_lg, pol), n_b)
    del hid

    achieved = eff_flops / (kernel_ms * 1e-3) / 1e12
    peak = MFMA_FP8_PEAK_TFLOPS if fp8kv else MFMA_BF16_PEAK_TFLOPS
    kernel_name = "k_attn_fp8" if fp8kv else "k_attn_bf16"
    traffic = measured_traffic_bytes(w.name, kernel_name) if args.layout == "appended" else None
    line = {
        "metric": "effective masked-attn TFLOP/s (unmasked FLOPs only), whole step: mask plan + attention + readout",
        "value": eff_flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "settle_ms": settle_ms, "settle_steps": settle_steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8" if fp8kv else "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layout": args.layout, "batch": pr.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "total_tokens": pr.total_tokens, "total_segments": pr.total_segments,
                   "rope_theta": w.rope_theta, "unmasked_pairs": pairs, "effective_flops": eff_flops,
                   "layers": 1},
        "pct_mfma_peak_step": 100.0 * eff_flops / (ms_per_step * 1e-3) / 1e12 / peak,
        "verified_prefixes_per_s": pr.total_segments / (ms_per_step * 1e-3),
        "breakdown_ms": {"pv_build_mask": t_build, "pv_masked_attention": t_attn, "pv_first_reject": t_read,
                         "attention_main_kernel": kernel_ms, "step_with_kernel_events": ms_per_step_events},
        "main_kernel_ms_series": kernel_series,
        "after_step_ms": {"pv_judge_logits_h4096": t_judge, "pv_decide": t_decide},
        "segment_rows_only": {"pv_segment_attention_ms": t_seg, "pv_prepare_kv_ms": t_prepare,
                              "pv_segment_attention_prepared_ms": t_seg_prepared, "unmasked_pairs": seg_pairs,
                              "tflops": (4.0 * w.head_dim * w.n_q_heads * seg_pairs / (t_seg * 1e-3) / 1e12) if t_seg else None},
        "attn_tflops": eff_flops / (t_attn * 1e-3) / 1e12,
        # the whole attention call (K/V preparation + main kernel) against the same peak, next to the
        # main kernel's own fraction in `roofline`
        "attention_call_frac": eff_flops / (t_attn * 1e-3) / 1e12 / peak,
        "max_abs_output": float(out.float().abs().max()),   # bf16 output spacing grows with |o|
        "roofline": {"bound": "mfma", "kernel": kernel_name, "achieved": achieved,
                     "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": traffic},
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, eff_flops)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
