"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, its pure host helpers agree with the oracle, and
argument errors are reported before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2509_00419_amd as lv
from oracle import lvlm_oracle as O
from paper_2509_00419_amd import binding as bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "lvlm.h")).read()
    declared = set(re.findall(r"LVLM_API[^;(]*?\b(lvlm_\w+)\s*\(", header))
    assert {"lvlm_score_tokens", "lvlm_merge_compact", "lvlm_kv_compress", "lvlm_decode_attn"} <= declared
    assert len(declared) >= 14 and "lvlm_merge_similar" in declared
    for name in declared:
        assert hasattr(bd.lib, name), name


def test_struct_sizes_match_the_header_layout():
    # natural alignment, no packing: sizes follow from the field lists in the header
    assert C.sizeof(bd.ScoreDesc) == 12 * 4 + 8 * 8
    assert C.sizeof(bd.Plane) == 2 * 8 + 2 * 8 + 4 * 4
    assert C.sizeof(bd.MergeDesc) == 6 * 4
    assert C.sizeof(bd.KvDesc) == 10 * 4 + 8
    assert C.sizeof(bd.AttnDesc) == 13 * 4


def test_schedule_helper_matches_oracle():
    for n_img, f, s in [(2048, 0.03, 3), (2048, 0.35, 3), (1792, 0.35, 3), (16384, 0.03, 3), (576, 0.5, 1),
                        (2048, 1.0, 3), (7, 0.001, 4)]:
        assert lv.schedule(n_img, f, s) == O.schedule(n_img, f, s)
    with pytest.raises(lv.LvlmError):
        lv.schedule(0, 0.5, 3)
    with pytest.raises(lv.LvlmError):
        lv.schedule(10, 0.0, 3)


def test_merge_weight_helper_matches_oracle():
    for mode in (lv.MERGE_LINEAR_RANK, lv.MERGE_PAIRWISE, lv.MERGE_LINEAR_RAW):
        for m in (1, 2, 5, 1413):
            got = lv.merge_weights(mode, m).numpy()
            np.testing.assert_allclose(got, O.merge_weights(mode, m).astype(np.float32), rtol=1e-7)


def _ctx():
    return lv.Context(0)       # creating a context touches no GPU state


def test_workspace_sizes_are_pure_host_arithmetic():
    ctx = _ctx()
    d = bd.ScoreDesc(bd.BF16, 1, 2176, 64, 2112, 28, 4, 128, 64, 2048, 1, 0.088, 28 * 128 * 64, 28 * 128, 128,
                     2176 * 512, 512, 128)
    assert ctx.workspace_bytes(bd.OP_SCORE, d) > 0
    kd = bd.KvDesc(bd.BF16, 16, 4, 128, 1056, 0, bd.KV_BUDGET, bd.ORDER_FILL, 1024, 1, 0.995)
    assert ctx.workspace_bytes(bd.OP_KV_COMPRESS, kd) >= 2 * 16 * 4 * 1056 * 4
    ad = bd.AttnDesc(bd.BF16, 16, 28, 4, 128, 1056, 1025, 2, 0, 0.088, 0.9)
    assert ctx.workspace_bytes(bd.OP_DECODE_ATTN, ad) > 0
    md = bd.MergeDesc(1, 2176, 64, 2048, 636, 1)
    planes = (bd.Plane * 1)(bd.Plane(0, 0, 2176 * 3584, 764 * 3584, 3584, bd.BF16, 0, 0))
    assert ctx.workspace_bytes(bd.OP_MERGE, bd.MergeQuery(C.pointer(md), planes)) > 2048 * 4


def test_argument_errors_are_reported_before_any_launch():
    ctx = _ctx()
    bad = bd.ScoreDesc(bd.BF16, 1, 100, 4, 96, 6, 4, 128, 0, 50, 1, 1.0, 0, 0, 128, 0, 0, 128)   # Hq % Hkv != 0
    with pytest.raises(lv.LvlmError) as e:
        ctx.workspace_bytes(bd.OP_SCORE, bad)
    assert e.value.status == 1 and "multiple" in str(e.value)
    bad = bd.ScoreDesc(bd.BF16, 1, 100, 4, 96, 4, 4, 96, 0, 50, 1, 1.0, 0, 0, 96, 0, 0, 96)       # head_dim 96
    with pytest.raises(lv.LvlmError):
        ctx.workspace_bytes(bd.OP_SCORE, bad)
    kd = bd.KvDesc(bd.BF16, 1, 1, 128, 64, 0, bd.KV_BUDGET, bd.ORDER_FILL, 0, 0, 0.5)              # budget 0
    with pytest.raises(lv.LvlmError):
        ctx.workspace_bytes(bd.OP_KV_COMPRESS, kd)
    # hot-path calls: null pointers, bad n_keep, missing workspace -- all fail on the host
    d = bd.ScoreDesc(bd.BF16, 1, 128, 4, 124, 4, 4, 128, 0, 64, 1, 1.0, 4 * 512, 512, 128, 128 * 512, 512, 128)
    st = bd.lib.lvlm_score_tokens(ctx._h, None, C.byref(d), None, None, None, None, None)
    assert st == 1 and b"null" in bd.lib.lvlm_last_error(ctx._h)
    st = bd.lib.lvlm_score_tokens(ctx._h, None, C.byref(d), 4096, 8192, None, 12288, 16384)
    assert st == 3 and b"workspace" in bd.lib.lvlm_last_error(ctx._h)
    st = bd.lib.lvlm_score_tokens(ctx._h, None, C.byref(d), 4100, 8192, None, 12288, 16384)
    assert st == 1 and b"aligned" in bd.lib.lvlm_last_error(ctx._h)
    md = bd.MergeDesc(1, 100, 10, 50, 51, 1)                                                       # n_keep > n_img
    planes = (bd.Plane * 1)(bd.Plane(4096, 1 << 20, 100 * 8, 100 * 8, 8, bd.BF16, 0, 0))
    st = bd.lib.lvlm_merge_compact(ctx._h, None, C.byref(md), 256, None, planes, None, None)
    assert st == 1 and b"n_keep" in bd.lib.lvlm_last_error(ctx._h)
    md = bd.MergeDesc(1, 100, 10, 50, 20, 1)
    planes = (bd.Plane * 1)(bd.Plane(4096, 4096 + 64, 100 * 8, 100 * 8, 8, bd.BF16, 0, 0))        # overlap
    st = bd.lib.lvlm_merge_compact(ctx._h, None, C.byref(md), 256, None, planes, None, None)
    assert st == 1 and b"overlap" in bd.lib.lvlm_last_error(ctx._h)
    planes = (bd.Plane * 1)(bd.Plane(4096, 1 << 20, 100 * 8, 100 * 8, 8, bd.I32, 0, 0))           # int + weighted
    st = bd.lib.lvlm_merge_compact(ctx._h, None, C.byref(md), 256, None, planes, None, None)
    assert st == 1 and b"integer" in bd.lib.lvlm_last_error(ctx._h)
    ad = bd.AttnDesc(bd.BF16, 1, 32, 2, 128, 64, 0, 2, 0, 1.0, 1.0)                                 # G = 16
    st = bd.lib.lvlm_decode_attn(ctx._h, None, C.byref(ad), 256, None, None, 512, 768, None, None, None, 1024, 2048)
    assert st == 2
    ad = bd.AttnDesc(bd.BF16, 1, 4, 2, 128, 64, 0, 2, 0, 1.0, 1.0)
    st = bd.lib.lvlm_decode_attn(ctx._h, None, C.byref(ad), 256, 512, None, 512, 768, None, None, None, 1024, 2048)
    assert st == 1 and b"together" in bd.lib.lvlm_last_error(ctx._h)


def test_score_plan_reports_the_launch_form():
    """lvlm_score_plan is the library's own launch decision (bench.py asks it instead of restating the rule)."""
    ctx = _ctx()

    def form(B, N, T, Hq, Hkv, n_img):
        d = bd.ScoreDesc(bd.BF16, B, N, T, N - T, Hq, Hkv, 128, 0, n_img, 1, 0.088, T * Hq * 128, Hq * 128, 128,
                         N * Hkv * 128, Hkv * 128, 128)
        return ctx.score_plan(d)

    assert form(1, 2176, 64, 28, 4, 2048) == 0             # one sequence of config 2's length: two passes
    assert form(1, 4608, 512, 32, 8, 4096) == 0            # 64 query chunks per KV head (more than a workgroup's waves hold in turn)
    assert form(1, 16512, 128, 48, 8, 16384) == 3          # one long sequence: the shared-tile kernel, keys in sixteen runs
    assert form(1, 845, 64, 28, 4, 717) == 1               # one short sequence: one launch, a chunk per workgroup
    assert form(64, 986, 96, 32, 8, 890) == 2              # many short sequences: shared key tiles
    assert form(12, 5219, 128, 48, 8, 5091) == 3           # 2.25 workgroups per compute unit over 5219 keys: keys in runs
    assert form(12, 1710, 128, 48, 8, 1582) == 2           # the same count over 1710 keys: too short to cut
    assert form(16, 5219, 128, 48, 8, 5091) == 2           # three workgroups per compute unit: nothing to even out
    bad = bd.ScoreDesc(bd.BF16, 1, 100, 4, 96, 6, 4, 128, 0, 50, 1, 1.0, 0, 0, 128, 0, 0, 128)
    with pytest.raises(lv.LvlmError):
        ctx.score_plan(bad)


def test_decode_plan_reports_the_split_of_a_launch():
    """lvlm_decode_plan is the library's own cut of a decode launch: one round of workgroups, whole 32-entry tiles, the
    steady-state shape (budget + 1 entries) as whole 128-entry splits plus one entry, and splits of ONE tile per wave
    wherever 128-entry splits are at most 1024 workgroups (bf16)."""
    ctx = _ctx()

    def plan(B, Hq, Hkv, Lmax, bound, dtype=bd.BF16, hd=128):
        return ctx.decode_plan(bd.AttnDesc(dtype, B, Hq, Hkv, hd, Lmax, bound, 2, 0, 0.088, 0.9))

    assert plan(16, 28, 4, 1152, 1025) == (8, 128, 2)             # config 4: 64 heads, budget 1024 + 1
    assert plan(1, 48, 8, 16640, 2049) == (16, 128, 2)            # config 5, steady state
    assert plan(8, 32, 8, 2048, 1889) == (15, 128, 0)             # config 3's longest layers: 960 one-tile workgroups
    assert plan(8, 32, 8, 2048, 1360) == (11, 128, 0)
    assert plan(8, 32, 8, 2048, 987) == (8, 128, 0)
    assert plan(8, 32, 8, 4096, 3000) == (8, 384, 1)              # 24 x 64 > 1024 workgroups: eight splits of three tiles
    assert plan(8, 32, 8, 2048, 1889, dtype=bd.F32) == (8, 256, 1)     # the fp32 kernel keeps one round of 512
    assert plan(8, 32, 8, 2048, 1820) == (15, 128, 0)             # a remainder of one tile no longer makes a two-tile launch
    assert plan(1, 48, 8, 16640, 16513)[0] == 58                  # 8 heads: at most 64 splits, here of 288 entries
    assert plan(1, 28, 4, 2304, 2178) == (17, 128, 1)             # one sequence: two entries past 17 whole splits go to one wave
    assert plan(1, 28, 4, 2304, 2240) == (18, 128, 0)             # ... a longer remainder is a split of its own
    for B, Hq, Hkv, Lmax, bound in ((3, 12, 4, 700, 0), (2, 8, 8, 129, 129), (1, 4, 1, 40000, 33000), (64, 32, 8, 520, 513)):
        n, sl, form = plan(B, Hq, Hkv, Lmax, bound)
        L = bound or Lmax
        assert 1 <= n <= 64 and sl % 32 == 0 and sl >= 128 and form in (0, 1, 2)
        assert n * sl >= L - (32 if form == 1 and sl == 128 else (1 if form == 2 else 0))
    with pytest.raises(lv.LvlmError):
        plan(1, 6, 4, 128, 0)                                      # heads not a multiple of KV heads


def test_size_arithmetic_survives_extreme_shapes():
    """Sizes at the documented limits are answered, sizes beyond them are refused -- and neither may overflow
    anything on the way (this file runs a second time against a build whose host code traps on signed overflow
    and other undefined behaviour)."""
    ctx = _ctx()
    big = 1 << 30

    def ask(op, d):
        n = C.c_size_t()
        st = bd.lib.lvlm_workspace_bytes(ctx._h, op, C.byref(d), C.byref(n))
        return st, n.value

    def score_desc(B, N, T, Hq, Hkv):
        n_img = max(1, N - T) if N > T else 1
        return bd.ScoreDesc(bd.BF16, B, N, T, max(0, N - T), Hq, Hkv, 128, 0, n_img, 1, 0.088, T * Hq * 128, Hq * 128, 128,
                            N * Hkv * 128, Hkv * 128, 128)

    # at the limits: B 65536, heads 1024, N 2^22, Lmax 2^24, row_elems 2^20
    for B, N, T, Hq, Hkv in ((65536, 1 << 22, 8191, 1024, 128), (65536, 1 << 22, 63, 1024, 1), (1, 1 << 22, 65535, 1024, 1024),
                             (65536, 1, 1, 8, 8)):
        st, n = ask(bd.OP_SCORE, score_desc(B, N, T, Hq, Hkv))
        assert st == 0 and n > 0, (B, N, T, Hq, Hkv)
        form = C.c_int32()
        assert bd.lib.lvlm_score_plan(ctx._h, C.byref(score_desc(B, N, T, Hq, Hkv)), C.byref(form)) == 0
    for B, H, Lmax in ((65536, 1024, 1 << 24), (1, 1, 1 << 24), (65536, 128, 1)):
        assert ask(bd.OP_KV_COMPRESS, bd.KvDesc(bd.BF16, B, H, 128, Lmax, 0, bd.KV_BUDGET, bd.ORDER_FILL, 1024, 1, 0.995))[0] == 0
        assert ask(bd.OP_KV_COMPRESS, bd.KvDesc(bd.F32, B, H, 64, Lmax, Lmax, bd.KV_THRESHOLD, bd.ORDER_STABLE, 0, 0, 0.5))[0] == 0
        Hq = min(8 * H, 1024)
        assert ask(bd.OP_DECODE_ATTN, bd.AttnDesc(bd.BF16, B, Hq, Hq // 8 if Hq >= 8 else Hq, 128, Lmax, 0, 2, 0, 0.088, 0.9))[0] == 0
        assert ask(bd.OP_DECODE_ATTN, bd.AttnDesc(bd.F32, B, H, H, 64, Lmax, Lmax, 2, 0, 0.088, 0.9,
                                                  Lmax - 1 if Lmax > 1 else 0, 1))[0] == 0
    for B, N, n_img, n_keep, C_ in ((65536, 1 << 22, 1 << 22, 1, 1 << 20), (1, 1 << 22, (1 << 22) - 5, 1 << 21, 8),
                                    (1, 17000, 16384, 5091, 6144)):
        md = bd.MergeDesc(B, N, 0, n_img, n_keep, 1)
        planes = (bd.Plane * 1)(bd.Plane(0, 0, N * C_, N * C_, C_, bd.BF16, 0, 0))
        assert ask(bd.OP_MERGE, bd.MergeQuery(C.pointer(md), planes))[0] == 0
        assert ask(bd.OP_MERGE_SIMILAR, bd.MergeQuery(C.pointer(md), planes))[0] == 0
    # beyond them: refused, with the limits in the message
    assert ask(bd.OP_SCORE, score_desc(1, big, 128, 48, 8))[0] == 1 and b"limits" in bd.lib.lvlm_last_error(ctx._h)
    assert ask(bd.OP_SCORE, score_desc(2 ** 31 - 1, 2 ** 31 - 1, 1, 2 ** 31 - 1, 1))[0] == 1
    assert ask(bd.OP_KV_COMPRESS, bd.KvDesc(bd.BF16, 2 ** 31 - 1, 2 ** 31 - 1, 128, 2 ** 31 - 1, 0, bd.KV_BUDGET, bd.ORDER_FILL,
                                            1024, 1, 0.995))[0] == 1
    assert ask(bd.OP_DECODE_ATTN, bd.AttnDesc(bd.BF16, 1, 8, 8, 128, 2 ** 31 - 1, 0, 2, 0, 0.088, 0.9))[0] == 1
    md = bd.MergeDesc(2 ** 31 - 1, 2 ** 31 - 1, 0, 2 ** 31 - 1, 1, 1)
    planes = (bd.Plane * 1)(bd.Plane(0, 0, 0, 0, 2 ** 31 - 1, bd.BF16, 0, 0))
    assert ask(bd.OP_MERGE, bd.MergeQuery(C.pointer(md), planes))[0] == 1
    for m in (1, 2, 100000):
        assert lv.merge_weights(lv.MERGE_LINEAR_RANK, m).numel() == m
    assert lv.schedule(2 ** 31 - 1, 0.5, 8)[-1] > 0
