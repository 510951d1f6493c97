"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes as C
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
pv = pytest.importorskip("paper_2605_04263_amd.binding")


def declared_functions():
    text = (ROOT / "include" / "pv.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pv_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"pv_build_mask", "pv_masked_attention", "pv_first_reject", "pv_query_sizes"} <= set(names)
    raw = C.CDLL(pv.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert pv.lib.pv_version().decode().startswith("pv ")
    assert pv.lib.pv_strerror(pv.PV_ERR_BOUNDARY).decode() != pv.lib.pv_strerror(pv.PV_OK).decode()


def q(problem, hq=8, hkv=2, d=128, dt=pv.PV_BF16):
    out = pv.PvSizes()
    st = pv.lib.pv_query_sizes(C.byref(problem.struct), hq, hkv, d, dt, C.byref(out))
    return st, out


def test_query_sizes_values():
    p = pv.make_problem([512], [2048], [16], [32], list(range(100, 1700, 100)))
    st, s = q(p, 32, 8, 128)
    assert st == pv.PV_OK
    assert s.total_tokens == 512 + 2048 + 16 * 32 == 3072       # T + n*|suffix| (+ prompt)
    assert s.total_segments == 16 and s.batch == 1 and s.max_seq_len == 3072
    assert s.n_q_tiles == 3072 // s.tile_m
    assert s.padded_keys == 3072
    assert s.dense_mask_bytes == 3072 * 3072
    assert s.plan_bytes > 4 * 3 * 3072 and s.plan_bytes % 16 == 0
    assert s.attn_workspace_bytes >= 2 * 8 * 3072 * 128 * 2
    # ragged: per-request rounding
    p = pv.make_problem([3, 0], [30, 70], [2, 0], [5, 1], [4, 30])
    st, s = q(p)
    assert st == pv.PV_OK
    assert s.total_tokens == 43 + 70 and s.max_seq_len == 70
    assert s.n_q_tiles == -(-43 // s.tile_m) + -(-70 // s.tile_m)
    assert s.padded_keys == 64 + 128
    assert s.dense_mask_bytes == 43 * 43 + 70 * 70


@pytest.mark.parametrize("args,expect", [
    (dict(hq=8, hkv=3), pv.PV_ERR_SHAPE),         # Hq % Hkv != 0
    (dict(hq=18, hkv=2), pv.PV_ERR_SHAPE),        # group of 9 > 8
    (dict(d=96), pv.PV_ERR_SHAPE),                # unsupported head_dim
    (dict(dt=7), pv.PV_ERR_DTYPE),
])
def test_head_validation(args, expect):
    p = pv.make_problem([4], [16], [2], [3], [5, 9])
    assert q(p, **args)[0] == expect


@pytest.mark.parametrize("fields,expect", [
    (([4], [16], [2], [3], [9, 5]), pv.PV_ERR_BOUNDARY),      # decreasing
    (([4], [16], [2], [3], [5, 17]), pv.PV_ERR_BOUNDARY),     # beyond the draft
    (([4], [16], [2], [3], [-1, 5]), pv.PV_ERR_BOUNDARY),
    (([4], [0], [0], [1], []), pv.PV_ERR_SHAPE),              # empty draft
    (([-1], [16], [0], [1], []), pv.PV_ERR_SHAPE),
    (([4], [16], [-2], [1], []), pv.PV_ERR_SHAPE),
    (([4], [16], [1], [0], [3]), pv.PV_ERR_SHAPE),            # empty segments
])
def test_problem_validation(fields, expect):
    assert q(pv.make_problem(*fields))[0] == expect


def test_boundaries_restart_per_request_and_duplicates_allowed():
    # second request's first boundary may be smaller than the first request's last one
    assert q(pv.make_problem([4, 4], [16, 16], [2, 2], [3, 3], [5, 9, 0, 0]))[0] == pv.PV_OK
    assert q(pv.make_problem([0], [16], [3], [1], [16, 16, 16]))[0] == pv.PV_OK


def test_null_pointers():
    out = pv.PvSizes()
    assert pv.lib.pv_query_sizes(None, 8, 2, 128, 0, C.byref(out)) == pv.PV_ERR_NULL
    p = pv.make_problem([4], [16], [2], [3], [5, 9])
    assert pv.lib.pv_query_sizes(C.byref(p.struct), 8, 2, 128, 0, None) == pv.PV_ERR_NULL
    broken = pv.PvProblem(1, None, None, None, None, None)
    assert pv.lib.pv_query_sizes(C.byref(broken), 8, 2, 128, 0, C.byref(out)) == pv.PV_ERR_NULL


def test_launch_calls_reject_bad_arguments_before_touching_the_gpu():
    p = pv.make_problem([4], [16], [2], [3], [5, 9])
    st, s = q(p, 8, 2, 128)
    assert st == pv.PV_OK
    fake = 0x1000                              # never dereferenced on these paths
    L = pv.lib
    assert L.pv_build_mask(C.byref(p.struct), C.byref(s), None, s.plan_bytes, None, 0, None) == pv.PV_ERR_NULL
    assert L.pv_build_mask(C.byref(p.struct), C.byref(s), fake, s.plan_bytes - 4, None, 0, None) == pv.PV_ERR_WORKSPACE
    assert L.pv_build_mask(C.byref(p.struct), C.byref(s), fake, s.plan_bytes, fake, 10, None) == pv.PV_ERR_WORKSPACE
    assert L.pv_build_mask(C.byref(p.struct), C.byref(s), fake + 4, s.plan_bytes, None, 0, None) == pv.PV_ERR_ALIGN
    other = pv.make_problem([4], [17], [2], [3], [5, 9])
    assert L.pv_build_mask(C.byref(other.struct), C.byref(s), fake, s.plan_bytes, None, 0, None) == pv.PV_ERR_SHAPE
    bad = pv.make_problem([4], [16], [2], [3], [9, 5])
    assert L.pv_build_mask(C.byref(bad.struct), C.byref(s), fake, s.plan_bytes, None, 0, None) == pv.PV_ERR_BOUNDARY

    att = lambda **kw: L.pv_masked_attention(
        C.byref(kw.get("s", s)), kw.get("plan", fake), kw.get("q", fake), fake, fake, kw.get("out", fake),
        None, kw.get("odt", pv.PV_BF16), kw.get("scale", 0.0), kw.get("theta", 0.0), kw.get("ws", fake),
        kw.get("wsb", s.attn_workspace_bytes), None)
    assert att(q=None) == pv.PV_ERR_NULL
    assert att(ws=None) == pv.PV_ERR_NULL
    assert att(wsb=s.attn_workspace_bytes - 1) == pv.PV_ERR_WORKSPACE
    assert att(out=fake + 2) == pv.PV_ERR_ALIGN
    assert att(odt=3) == pv.PV_ERR_DTYPE
    assert att(scale=-1.0) == pv.PV_ERR_SHAPE
    assert att(theta=float("nan")) == pv.PV_ERR_SHAPE
    tampered = pv.PvSizes.from_buffer_copy(s)
    tampered.plan_bytes += 16
    assert att(s=tampered) == pv.PV_ERR_SHAPE
    # a hand-made sizes struct beyond the documented limits is refused even if its plan size agrees
    huge = pv.PvSizes.from_buffer_copy(s)
    huge.total_tokens = (1 << 27) + 64
    huge.padded_keys = (1 << 27) + 64
    assert att(s=huge) == pv.PV_ERR_SHAPE
    many = pv.PvSizes.from_buffer_copy(s)
    many.total_segments = s.total_tokens + 1
    assert att(s=many) == pv.PV_ERR_SHAPE
    st, s32 = q(p, 8, 2, 128, pv.PV_F32)
    assert att(s=s32, odt=pv.PV_BF16, wsb=s32.attn_workspace_bytes) == pv.PV_ERR_DTYPE   # fp32 in needs fp32 out

    assert L.pv_first_reject(C.byref(s), fake, None, 0.0, 0, fake, None) == pv.PV_ERR_NULL
    assert L.pv_first_reject(C.byref(s), fake, fake, 0.0, 2, fake, None) == pv.PV_ERR_SHAPE
    assert L.pv_first_reject(C.byref(s), fake, fake, float("nan"), 0, fake, None) == pv.PV_ERR_SHAPE
    assert L.pv_first_reject(C.byref(s), None, fake, 0.0, 0, fake, None) == pv.PV_ERR_NULL
    assert L.pv_plan_export(C.byref(s), None, None, None, None, None, None) == pv.PV_ERR_NULL
    assert L.pv_profile_read(None) == pv.PV_ERR_NULL


def test_policy_calls_reject_bad_arguments_before_touching_the_gpu():
    p = pv.make_problem([4], [16], [2], [3], [5, 9])
    st, s = q(p, 8, 2, 128)
    assert st == pv.PV_OK
    fake = 0x1000
    L = pv.lib
    pol = pv.make_policy(4.0, 2.0, 6.0, 3.0, [3.0, 3.0], 0.3, 2, 0.0)
    dec = lambda **kw: L.pv_decide(C.byref(s), kw.get("plan", fake), kw.get("lg", fake), kw.get("full", fake),
                                   C.byref(kw["pol"]) if kw.get("pol") is not None else None,
                                   kw.get("out", fake), None)
    assert dec(pol=None) == pv.PV_ERR_NULL
    assert dec(pol=pol, lg=None) == pv.PV_ERR_NULL
    assert dec(pol=pol, full=None) == pv.PV_ERR_NULL              # full-answer logits needed outside premature mode
    assert dec(pol=pol, out=fake + 4) == pv.PV_ERR_ALIGN
    bad = pv.make_policy(4.0, 2.0, 6.0, 3.0, [3.0], 0.3, -1, 0.0)
    assert dec(pol=bad) == pv.PV_ERR_SHAPE
    bad = pv.make_policy(4.0, 2.0, 6.0, 3.0, [3.0], 0.3, 2, -0.5)
    assert dec(pol=bad) == pv.PV_ERR_SHAPE
    bad = pv.make_policy(float("nan"), 2.0, 6.0, 3.0, [3.0], 0.3, 2, 0.0)
    assert dec(pol=bad) == pv.PV_ERR_SHAPE
    bad = pv.make_policy(4.0, 2.0, 6.0, 3.0, [3.0], 0.3, 2, 0.0)
    bad.n_short = 9
    assert dec(pol=bad) == pv.PV_ERR_SHAPE

    jl = lambda **kw: L.pv_judge_logits(C.byref(s), kw.get("plan", fake), kw.get("h", fake), kw.get("w", fake),
                                        kw.get("hs", 64), kw.get("out", fake), None)
    assert jl(h=None) == pv.PV_ERR_NULL
    assert jl(hs=60) == pv.PV_ERR_SHAPE
    assert jl(hs=0) == pv.PV_ERR_SHAPE
    assert jl(w=fake + 2) == pv.PV_ERR_ALIGN
    assert jl(plan=None) == pv.PV_ERR_NULL


def test_layout_is_validated_and_sized():
    args = ([4], [16], [2], [3], [5, 9])
    st, s0 = q(pv.make_problem(*args), 8, 2, 128)
    inter = pv.make_problem(*args, layout=pv.PV_LAYOUT_INTERLEAVED)
    st1, s1 = q(inter, 8, 2, 128)
    assert st == st1 == pv.PV_OK
    assert s1.layout == pv.PV_LAYOUT_INTERLEAVED and s0.layout == pv.PV_LAYOUT_APPENDED
    assert s1.plan_bytes >= s0.plan_bytes + 4 * s0.total_tokens        # the row map
    assert (s1.total_tokens, s1.n_q_tiles, s1.padded_keys) == (s0.total_tokens, s0.n_q_tiles, s0.padded_keys)
    bad = pv.make_problem(*args, layout=2)
    assert q(bad, 8, 2, 128)[0] == pv.PV_ERR_SHAPE
    fake = 0x1000
    # sizes of one layout with a problem of the other: refused before any launch
    assert pv.lib.pv_build_mask(C.byref(inter.struct), C.byref(s0), fake, s1.plan_bytes, None, 0, None) == pv.PV_ERR_SHAPE
    tampered = pv.PvSizes.from_buffer_copy(s0)
    tampered.layout = pv.PV_LAYOUT_INTERLEAVED                         # plan_bytes no longer matches
    assert pv.lib.pv_first_reject(C.byref(tampered), fake, fake, 0.0, 0, fake, None) == pv.PV_ERR_SHAPE


def test_segment_attention_validates_like_the_full_call():
    p = pv.make_problem([4], [16], [2], [3], [5, 9])
    st, s = q(p, 8, 2, 128)
    assert st == pv.PV_OK and s.n_seg_tiles == 1                      # rows 20..25 sit in tile 0
    fake = 0x1000
    seg = lambda **kw: pv.lib.pv_segment_attention(
        C.byref(kw.get("s", s)), fake, kw.get("q", fake), fake, fake, kw.get("out", fake), None,
        kw.get("odt", pv.PV_BF16), 0.0, 0.0, fake, kw.get("wsb", s.attn_workspace_bytes), None)
    assert seg(q=None) == pv.PV_ERR_NULL
    assert seg(out=fake + 2) == pv.PV_ERR_ALIGN
    assert seg(wsb=s.attn_workspace_bytes - 1) == pv.PV_ERR_WORKSPACE   # the partial results are part of it
    st, s32 = q(p, 8, 2, 128, pv.PV_F32)
    assert seg(s=s32, odt=pv.PV_F32, wsb=s32.attn_workspace_bytes) == pv.PV_ERR_DTYPE   # bf16 inputs only
    tampered = pv.PvSizes.from_buffer_copy(s)
    tampered.n_seg_tiles = 2
    assert seg(s=tampered) == pv.PV_ERR_SHAPE
    # a request without segments has no such tile; one whose segments start on a tile border has its own
    assert q(pv.make_problem([4], [16], [0], [3], []), 8, 2, 128)[1].n_seg_tiles == 0
    assert q(pv.make_problem([32], [32], [2], [40], [5, 9]), 8, 2, 128)[1].n_seg_tiles == 3


def test_margin_from_tau_host_call():
    # the margin whose two-way confidence is tau: checked by putting it back through the logistic
    # function with 60 digits, for the thresholds of the paper's hyper-parameter table
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    golden = ROOT / "tests" / "golden" / "judge_thresholds.txt"
    taus = [x for x in golden.read_text().split("\n") if x and not x.startswith("#")]
    assert len(taus) >= 7
    for t in taus:
        m = pv.pv_margin_from_tau(float(t))
        conf = 1 / (1 + (-Decimal(m)).exp())
        assert abs(conf - Decimal(float(t))) < Decimal("1e-15"), (t, m)
    assert pv.pv_margin_from_tau(0.5) == 0.0
    out = C.c_double(7.0)
    for bad in (0.0, 1.0, -0.1, 1.5, float("nan")):
        assert pv.lib.pv_margin_from_tau(bad, C.byref(out)) == pv.PV_ERR_SHAPE
    assert pv.lib.pv_margin_from_tau(0.9, None) == pv.PV_ERR_NULL
    assert out.value == 7.0


def test_prepared_key_calls_validate_on_the_host():
    p = pv.make_problem([4], [60], [2], [3], [5, 9])
    st, s = q(p, 8, 2, 128)
    assert st == pv.PV_OK
    fake = 0x1000
    L = pv.lib
    prep = lambda **kw: L.pv_prepare_kv(C.byref(kw.get("s", s)), fake, kw.get("k", fake), fake, kw.get("bt", None),
                                        kw.get("ps", 0), kw.get("first", 0), kw.get("last", s.total_tokens),
                                        kw.get("cap", 0), 0.0, kw.get("ws", fake),
                                        kw.get("wsb", s.attn_workspace_bytes), None)
    assert prep(k=None) == pv.PV_ERR_NULL
    assert prep(ws=None) == pv.PV_ERR_NULL
    assert prep(first=-1) == pv.PV_ERR_SHAPE
    assert prep(first=9, last=8) == pv.PV_ERR_SHAPE
    assert prep(last=s.total_tokens + 1) == pv.PV_ERR_SHAPE
    assert prep(bt=fake, ps=0) == pv.PV_ERR_SHAPE                       # a block table needs a page size
    assert prep(bt=fake + 2, ps=16) == pv.PV_ERR_ALIGN
    assert prep(cap=s.padded_keys - 64) == pv.PV_ERR_SHAPE              # capacity below this plan's keys
    assert prep(cap=s.padded_keys + 32) == pv.PV_ERR_SHAPE              # not a multiple of the key tile
    assert prep(wsb=s.attn_workspace_bytes - 1) == pv.PV_ERR_WORKSPACE
    st32, s32 = q(p, 8, 2, 128, pv.PV_F32)
    assert prep(s=s32, wsb=s32.attn_workspace_bytes) == pv.PV_ERR_DTYPE  # bf16 inputs only
    # workspace for a larger head stride: grows with the capacity, equals the ordinary size for 0
    assert pv.pv_prepared_workspace_bytes(s, 0) == s.attn_workspace_bytes
    big = pv.pv_prepared_workspace_bytes(s, s.padded_keys + 640)
    assert big >= s.attn_workspace_bytes + 2 * 2 * 640 * 128 * 2
    assert prep(cap=s.padded_keys + 640, wsb=big - 1) == pv.PV_ERR_WORKSPACE
    att = lambda **kw: L.pv_segment_attention_prepared(C.byref(s), fake, kw.get("q", fake), fake, fake, None, 0,
                                                       kw.get("cap", 0), kw.get("out", fake), None, pv.PV_BF16,
                                                       0.0, 0.0, fake, s.attn_workspace_bytes, None)
    assert att(q=None) == pv.PV_ERR_NULL
    assert att(out=None) == pv.PV_ERR_NULL
    assert att(cap=-64) == pv.PV_ERR_SHAPE
    # the count of short segment rows is part of the sizes (a segment that sees almost nothing)
    assert s.n_short_seg_rows == 6 and s.n_short_rows == 16 + 6         # 4 + 9 + 3 = 16 keys at most
    far = q(pv.make_problem([4], [60], [2], [3], [30, 60]), 8, 2, 128)[1]
    assert far.n_short_seg_rows == 0 and far.n_short_rows == 16
