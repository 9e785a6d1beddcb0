"""GPU parity: every entry point of the C ABI against the CPU oracle, element by
element, on the same seeded inputs.

Tolerances (max |gpu - oracle| / max |oracle|): 1e-5 for fp32 results (scores
are fp32 whatever the input dtype), 2e-2 for bf16 results.  Index lists, kept
sets, slot moves and lengths are compared exactly; where floating point feeds
an integer decision (which tokens are kept, which entries are evicted) the
oracle takes that decision on the GPU's own score bits.
"""
import math

import numpy as np
import pytest
import torch

import paper_2509_00419_amd as lv
from oracle import lvlm_oracle as O
from workloads import configs, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def f64(t):
    return t.detach().double().cpu().numpy()


def rel_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


@pytest.fixture(scope="module")
def ctx():
    return lv.Context(0)


def _rand(shape, dtype, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (scale * torch.randn(*shape, generator=g)).to(dtype)


# --------------------------------------------------------------------------- step 1: score
SCORE_CASES = [
    # dtype, B, T, Hq, Hkv, d, n_sys, n_img, causal           what it covers
    (torch.float32, 1, 32, 4, 4, 64, 32, 576, True),          # config 1
    (torch.float32, 2, 5, 4, 2, 128, 3, 70, True),            # fp32, d=128, ragged everything
    (torch.bfloat16, 1, 64, 28, 4, 128, 64, 2048, True),      # config 2 layer: G=7, 14 row chunks
    (torch.bfloat16, 2, 9, 6, 2, 128, 5, 333, True),          # G*T = 27 (< one chunk), ragged keys
    (torch.bfloat16, 1, 33, 8, 8, 64, 0, 200, False),         # d=64, no mask, no system prefix
    (torch.bfloat16, 3, 40, 14, 2, 128, 7, 1000, True),       # G=7 with T=40: 280 rows = 8.75 chunks
    # short sequences take both passes in one launch (one workgroup per 32-row chunk); the cases above with
    # N <= 1100 rows of 256 bytes are of that kind, the ones below keep the two-pass kernels on ragged shapes
    (torch.bfloat16, 1, 64, 28, 4, 128, 64, 717, True),       # config 2 after the first merge: 14 chunks, one launch
    (torch.bfloat16, 2, 9, 6, 2, 128, 5, 1500, True),         # two-pass, G*T = 27, ragged keys
    (torch.bfloat16, 1, 33, 8, 8, 64, 0, 2300, False),        # two-pass, d=64, no mask
    (torch.float32, 2, 5, 4, 2, 128, 3, 700, True),           # two-pass, fp32 d=128
]


@pytest.mark.parametrize("dtype,B,T,Hq,Hkv,d,n_sys,n_img,causal", SCORE_CASES)
def test_score_tokens(ctx, dtype, B, T, Hq, Hkv, d, n_sys, n_img, causal):
    N = n_sys + n_img + T
    q, k = _rand((B, T, Hq, d), dtype, 1), _rand((B, N, Hkv, d), dtype, 2)
    kw = dict(q_pos0=n_sys + n_img, img_begin=n_sys, n_img=n_img, causal=causal)
    sh, sm = ctx.score_tokens(q.to(DEV), k.to(DEV), **kw)
    osh, osm = O.score_tokens(f64(q), f64(k), **kw)
    assert rel_err(sh.cpu(), osh) < 1e-5
    assert rel_err(sm.cpu(), osm) < 1e-5
    # the caller-supplied row normaliser gives the same scores as the library's own pass
    tk = k.double().repeat_interleave(Hq // Hkv, dim=2)
    s = torch.einsum("bthd,bnhd->bhtn", q.double(), tk) / math.sqrt(d)
    if causal:
        mask = torch.arange(N)[None, :] > (n_sys + n_img + torch.arange(T))[:, None]
        s = s.masked_fill(mask, float("-inf"))
    lse = torch.logsumexp(s, dim=-1).float().contiguous()
    sh2, sm2 = ctx.score_tokens(q.to(DEV), k.to(DEV), row_lse=lse.to(DEV), **kw)
    assert rel_err(sh2.cpu(), osh) < 1e-5 and rel_err(sm2.cpu(), osm) < 1e-5


@pytest.mark.parametrize("B,T,Hq,Hkv,n_sys,n_img", [
    (4, 128, 48, 8, 0, 2072),        # 192 workgroups of four chunks: three quarters of a workgroup per compute unit
    (6, 100, 48, 8, 3, 2500),        # 19 chunks per KV head (the last workgroup of a head has three), image span from key 3
    (4, 128, 48, 8, 5, 3001),        # an odd number of image keys: the last run ends inside a tile
    (8, 100, 28, 4, 3, 3000),        # G = 7
])
def test_score_tokens_keys_in_runs(ctx, B, T, Hq, Hkv, n_sys, n_img):
    """Launches of few workgroups over long sequences cut the keys into runs (one launch per sweep, the runs' normaliser
    partials folded in between): the same scores, with the library's own normalisers and with the caller's, and with a
    logit far above the rest in a late run (the sweep that takes the first tile's maximum as reference must notice)."""
    d, N = 128, n_sys + n_img + T
    q, k = _rand((B, T, Hq, d), torch.bfloat16, 11), _rand((B, N, Hkv, d), torch.bfloat16, 12)
    kw = dict(q_pos0=n_sys + n_img, img_begin=n_sys, n_img=n_img, causal=True)
    assert ctx.score_plan(ctx.score_desc(q, k, **kw)) == 3
    for far in (False, True):
        if far:                                          # one key of one head lines up with a query row, 40 times as long
            k = k.clone()
            k[B - 1, n_sys + (7 * n_img) // 8, Hkv - 1] = (40.0 * q[B - 1, T // 2, Hq - 1].float()).to(torch.bfloat16)
        sh, sm = ctx.score_tokens(q.to(DEV), k.to(DEV), **kw)
        osh, osm = O.score_tokens(f64(q), f64(k), **kw)
        assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5, far
    tk = k.double().repeat_interleave(Hq // Hkv, dim=2)
    s = torch.einsum("bthd,bnhd->bhtn", q.double(), tk) / math.sqrt(d)
    mask = torch.arange(N)[None, :] > (n_sys + n_img + torch.arange(T))[:, None]
    lse = torch.logsumexp(s.masked_fill(mask, float("-inf")), dim=-1).float().contiguous()
    sh2, sm2 = ctx.score_tokens(q.to(DEV), k.to(DEV), row_lse=lse.to(DEV), **kw)
    assert rel_err(sh2.cpu(), osh) < 1e-5 and rel_err(sm2.cpu(), osm) < 1e-5


@pytest.mark.parametrize("N", [300, 1300])      # one launch for both passes / the two-pass kernels
def test_score_tokens_mask_inside_span_and_strided_inputs(ctx, N):
    # query rows start INSIDE the scored span (all-rows reading): the causal mask bites in pass 1 too;
    # q and k are views into wider buffers (non-trivial strides)
    B, T, H, d = 2, 48, 4, 128
    qkv = _rand((B, N, 3, H, d), torch.bfloat16, 3)
    q_all, k_all = qkv[:, :, 0], qkv[:, :, 1]
    q = q_all[:, N - T:]
    kw = dict(q_pos0=N - T, img_begin=10, n_img=N - 10, causal=True)
    qkv_d = qkv.to(DEV)
    q_d, k_d = qkv_d[:, N - T:, 0], qkv_d[:, :, 1]                 # strided views, not copies
    assert not q_d.is_contiguous() and not k_d.is_contiguous()
    sh, sm = ctx.score_tokens(q_d, k_d, **kw)
    osh, osm = O.score_tokens(f64(q), f64(k_all), **kw)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5
    assert float(sm[:, -1].max()) < 1.0                            # last key is seen by one row only


def test_score_all_rows_reading_long_sequence(ctx):
    # every row of the sequence is a query row (the all-rows reading of Sec. 3.2.1) under the causal mask: half
    # of the (key block, row chunk) pairs lie wholly above the diagonal and are skipped, the ones on it are
    # masked element by element; 2176 tokens, G = 4
    B, N, Hq, Hkv, d, n_sys, n_img = 1, 2176, 8, 2, 128, 64, 2048
    q, k = _rand((B, N, Hq, d), torch.bfloat16, 5), _rand((B, N, Hkv, d), torch.bfloat16, 6)
    kw = dict(q_pos0=0, img_begin=n_sys, n_img=n_img, causal=True)
    sh, sm = ctx.score_tokens(q.to(DEV), k.to(DEV), **kw)
    osh, osm = O.score_tokens(f64(q), f64(k), **kw)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5
    # an early image key is seen by almost every row, the last one by the text rows only
    assert float(sm[0, 0]) > float(sm[0, -1])


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_score_from_probs(ctx, dtype):
    # attention probabilities handed in (a plain attention's matrix): ragged sizes, G = 3, a strided view of a
    # wider buffer; and the config-2 shape (28/4 heads, 64 rows, 2176 keys)
    for B, T, Hq, Hkv, N, img0, n_img, seed in ((2, 37, 6, 2, 301, 5, 290, 7), (1, 64, 28, 4, 2176, 64, 2048, 8)):
        g = torch.Generator().manual_seed(seed)
        wide = torch.softmax(3.0 * torch.randn(B, Hq, T + 3, (N + 47) // 32 * 32, generator=g), dim=-1).to(dtype)
        p = wide[:, :, 2:2 + T, 8:8 + N]                      # rows and columns cut out of a larger array
        p_d = wide.to(DEV)[:, :, 2:2 + T, 8:8 + N]
        assert not p_d.is_contiguous()
        sh, sm = ctx.score_from_probs(p_d, n_kv_heads=Hkv, img_begin=img0, n_img=n_img)
        osh, osm = O.score_from_probs(f64(p), n_kv_heads=Hkv, img_begin=img0, n_img=n_img)
        assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5
    # the two sources of Sec. 3.2.2 agree: probabilities computed here give what lvlm_score_tokens computes itself
    B, T, Hq, Hkv, d, n_sys, n_img = 1, 32, 8, 4, 64, 16, 400
    N = n_sys + n_img + T
    q, k = _rand((B, T, Hq, d), dtype, 9), _rand((B, N, Hkv, d), dtype, 10)
    s = torch.einsum("bthd,bnhd->bhtn", q.double(), k.double().repeat_interleave(Hq // Hkv, dim=2)) / math.sqrt(d)
    mask = torch.arange(N)[None, :] > (n_sys + n_img + torch.arange(T))[:, None]
    probs = torch.softmax(s.masked_fill(mask, float("-inf")), dim=-1).float().contiguous()
    a_h, a_m = ctx.score_from_probs(probs.to(DEV), n_kv_heads=Hkv, img_begin=n_sys, n_img=n_img)
    b_h, b_m = ctx.score_tokens(q.to(DEV), k.to(DEV), q_pos0=n_sys + n_img, img_begin=n_sys, n_img=n_img)
    assert rel_err(a_h.cpu(), b_h.cpu()) < 1e-5 and rel_err(a_m.cpu(), b_m.cpu()) < 1e-5


def test_score_batched_form_with_logits_far_above_the_first_tile(ctx):
    # 32 sequences x 8 KV heads, three query chunks each: the one-launch form whose workgroups share the key tiles.
    # Its first sweep keeps the first tile's reference; keys whose logits lie far above everything before them
    # (natural-log distance 120) must send the workgroup through the careful sweep, others not.
    B, T, Hq, Hkv, d, n_sys, n_img = 32, 96, 8, 8, 64, 8, 280
    N = n_sys + n_img + T
    g = torch.Generator().manual_seed(21)
    q = 0.05 * torch.randn(B, T, Hq, d, generator=g)
    k = 0.05 * torch.randn(B, N, Hkv, d, generator=g)
    q[:, :, 0:3, 0] = 22.0
    k[:, :, 0:3, 0] = -22.0
    k[:, 100:130, 0:3, 0] = 22.0
    k[:, 200, 1, 0] = 30.0
    q, k = q.bfloat16(), k.bfloat16()
    kw = dict(q_pos0=n_sys + n_img, img_begin=n_sys, n_img=n_img)
    sh, sm = ctx.score_tokens(q.to(DEV), k.to(DEV), **kw)
    osh, osm = O.score_tokens(f64(q), f64(k), **kw)
    assert torch.isfinite(sh).all()
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5


def test_score_wide_blocks_config3_shape(ctx):
    # B=8, 8 KV heads, N=1888: enough workgroups for the 256-key blocks (2 tiles per wave)
    w = configs.CFG3
    x = synth.layer_inputs(w, with_v=False)
    kw = dict(q_pos0=w.n_sys + w.n_img, img_begin=w.n_sys, n_img=w.n_img)
    sh, sm = ctx.score_tokens(x["q"].to(DEV), x["k"].to(DEV), **kw)
    osh, osm = O.score_tokens(f64(x["q"]), f64(x["k"]), **kw)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5


# --------------------------------------------------------------------------- steps 2-4
def _merge_case(ctx, dtype, B, n_sys, n_img, n_txt, C, n_keep, score=None, w_mode=None, extra_planes=True, seed=0):
    N = n_sys + n_img + n_txt
    hid = _rand((B, N, C), dtype, seed + 10)
    if score is None:
        score = torch.rand(B, n_img, generator=torch.Generator().manual_seed(seed + 11))
    planes, rules, dts = [hid], [lv.RULE_WEIGHTED], ["bf16" if dtype == torch.bfloat16 else "f32"]
    if extra_planes:
        planes += [_rand((B, N, 24), dtype, seed + 12), torch.arange(B * N * 3, dtype=torch.int32).view(B, N, 3),
                   torch.arange(B * N, dtype=torch.int32).view(B, N, 1)]
        rules += [lv.RULE_WEIGHTED, lv.RULE_TOP, lv.RULE_TOP]
        dts += [dts[0], "f32", "f32"]
    r = n_img - n_keep
    w = None if w_mode is None else lv.merge_weights(w_mode, r + 1)
    outs, keep, merged = ctx.merge_compact([p.to(DEV) for p in planes], score.to(DEV), img_begin=n_sys,
                                           n_img=n_img, n_keep=n_keep, rules=rules,
                                           w=None if w is None else w.to(DEV))
    np_planes = [f64(p) if p.dtype != torch.int32 else p.numpy() for p in planes]
    oouts, okeep, omerged = O.merge_compact(np_planes, score.numpy(), img_begin=n_sys, n_img=n_img, n_keep=n_keep,
                                            rules=rules, dtypes=dts, w=None if w is None else w.numpy())
    if r > 0:
        assert np.array_equal(keep.cpu().numpy(), okeep)
        assert np.array_equal(merged.cpu().numpy(), omerged)
    for got, ref, p in zip(outs, oouts, planes):
        got = got.cpu()
        assert tuple(got.shape) == ref.shape
        if p.dtype == torch.int32:
            assert np.array_equal(got.numpy(), ref)
            continue
        got = f64(got)
        new_row = n_sys + n_keep - 1
        rest = np.ones(ref.shape[1], bool)
        if r > 0:
            rest[new_row] = False
            assert rel_err(got[:, new_row], ref[:, new_row]) < TOL[dtype]
        assert np.array_equal(got[:, rest], ref[:, rest])            # copied rows are bit-exact


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n_keep", [1, 2, 288, 575, 576])
def test_merge_compact_config1_sizes(ctx, dtype, n_keep):
    _merge_case(ctx, dtype, 1, 32, 576, 32, 256, n_keep)


def test_merge_compact_ragged_batch_and_tables(ctx):
    _merge_case(ctx, torch.bfloat16, 3, 5, 1333, 7, 520, 400, seed=1)                       # rows of 1040 B
    _merge_case(ctx, torch.bfloat16, 2, 0, 2500, 0, 3584, 99, extra_planes=False, seed=2)   # > 2 rank tiles
    _merge_case(ctx, torch.float32, 2, 3, 300, 4, 100, 120, w_mode=lv.MERGE_PAIRWISE, seed=3)
    _merge_case(ctx, torch.bfloat16, 1, 3, 300, 4, 257, 120, w_mode=lv.MERGE_LINEAR_RAW, seed=4)  # odd row: 2-byte units


def test_merge_compact_ties_and_special_scores(ctx):
    n_img = 700
    _merge_case(ctx, torch.float32, 1, 2, n_img, 2, 64, 300, score=torch.full((1, n_img), 0.25), seed=5)
    s = torch.rand(2, n_img, generator=torch.Generator().manual_seed(6))
    s = (s * 8).floor() / 8                                                              # heavy ties
    s[0, 5], s[0, 6], s[1, 7], s[1, 8] = float("nan"), float("-inf"), -0.0, float("inf")
    _merge_case(ctx, torch.float32, 2, 2, n_img, 2, 64, 123, score=s, seed=7)


@pytest.mark.parametrize("n_img", [8192, 8193, 9000, 17000])
def test_merge_compact_long_sequences_rank_by_sorted_blocks(ctx, n_img):
    # from 8192 image tokens on the ranks come from sorted blocks of 1024 tokens and binary searches instead of
    # counting: whole and ragged block counts, heavy ties (eight distinct scores), NaN / inf / signed zeros, two
    # sequences; the index lists must equal the oracle's, order included
    s = torch.rand(2, n_img, generator=torch.Generator().manual_seed(n_img))
    s[1] = (s[1] * 8).floor() / 8
    s[0, 5], s[0, 1030], s[1, 7], s[1, 2048], s[0, n_img - 1] = float("nan"), float("-inf"), -0.0, float("inf"), 0.0
    _merge_case(ctx, torch.bfloat16, 2, 2, n_img, 3, 64, n_img // 3, score=s, extra_planes=False, seed=n_img)
    if n_img == 8192:       # all scores equal: the order is the index order
        _merge_case(ctx, torch.float32, 1, 0, n_img, 0, 64, 100, score=torch.full((1, n_img), 0.5), extra_planes=False, seed=9)


def test_merge_compact_non_finite_rows_outside_p_merged(ctx):
    # Sec. 3.2.1: P_new = W_v x P_merged touches the r+1 merged rows only.  An inf / NaN in a kept image row, in a
    # text row or in a system row must be copied as it is and must not leak into the merged token.
    B, n_sys, n_img, n_txt, C, n_keep = 2, 3, 400, 5, 264, 150
    N = n_sys + n_img + n_txt
    for dtype in (torch.bfloat16, torch.float32):
        hid = _rand((B, N, C), dtype, 130)
        score = torch.rand(B, n_img, generator=torch.Generator().manual_seed(131))
        order = torch.argsort(score, dim=1, descending=True)
        for b in range(B):
            kept = order[b, :n_keep - 1]
            hid[b, n_sys + int(kept[0]), 7] = float("inf")
            hid[b, n_sys + int(kept[5]), 0] = float("nan")
            hid[b, n_sys + int(kept[-1]), C - 1] = float("-inf")
        hid[:, 1, 3] = float("inf")                      # a system row
        hid[:, N - 2, 100] = float("-inf")               # an instruction row
        (out,), keep, merged = ctx.merge_compact([hid.to(DEV)], score.to(DEV), img_begin=n_sys, n_img=n_img, n_keep=n_keep)
        (ref,), okeep, omerged = O.merge_compact([f64(hid)], score.numpy(), img_begin=n_sys, n_img=n_img, n_keep=n_keep,
                                                 dtypes=["bf16" if dtype == torch.bfloat16 else "f32"])
        assert np.array_equal(keep.cpu().numpy(), okeep) and np.array_equal(merged.cpu().numpy(), omerged)
        got = f64(out.cpu())
        new_row = n_sys + n_keep - 1
        assert np.isfinite(got[:, new_row]).all() and np.isfinite(ref[:, new_row]).all()
        assert rel_err(got[:, new_row], ref[:, new_row]) < TOL[dtype]
        rest = np.ones(ref.shape[1], bool)
        rest[new_row] = False
        assert np.array_equal(got[:, rest], ref[:, rest], equal_nan=True)      # copied rows bit for bit, inf and NaN too


def test_merge_compact_full_config2_stage_from_gpu_scores(ctx):
    # config 2, first merge layer at the 3 % schedule: 2048 -> 636, all planes a layer carries
    w = configs.CFG2
    x = synth.layer_inputs(w)
    n_keep = lv.schedule(w.n_img, 0.03, 3)[0]
    assert n_keep == 636
    _, sm = ctx.score_tokens(x["q"].to(DEV), x["k"].to(DEV), q_pos0=w.n_sys + w.n_img, img_begin=w.n_sys,
                             n_img=w.n_img)
    N = w.seq_len
    planes = [x["hidden"], x["k"].view(1, N, -1), x["v"].view(1, N, -1), x["pos"]]
    rules = [lv.RULE_WEIGHTED] * 3 + [lv.RULE_TOP]
    outs, keep, merged = ctx.merge_compact([p.to(DEV) for p in planes], sm, img_begin=w.n_sys, n_img=w.n_img,
                                           n_keep=n_keep, rules=rules)
    np_planes = [f64(p) for p in planes[:3]] + [planes[3].numpy()]
    oouts, okeep, omerged = O.merge_compact(np_planes, sm.cpu().numpy(), img_begin=w.n_sys, n_img=w.n_img,
                                            n_keep=n_keep, rules=rules, dtypes=["bf16"] * 3 + ["f32"])
    assert np.array_equal(keep.cpu().numpy(), okeep) and np.array_equal(merged.cpu().numpy(), omerged)
    assert outs[0].shape[1] == w.n_sys + 636 + w.n_text                                   # schedule count
    for got, ref in zip(outs[:3], oouts[:3]):
        assert rel_err(f64(got.cpu()), ref) < 2e-2
    assert np.array_equal(outs[3].cpu().numpy(), oouts[3])


# --------------------------------------------------------------------------- step 5
def _cache(dtype, B, H, Lmax, d, lens, seed, protected=4, dyadic=False, image_only=False, flat=False):
    g = torch.Generator().manual_seed(seed)
    k, v = _rand((B, H, Lmax, d), dtype, seed + 1), _rand((B, H, Lmax, d), dtype, seed + 2)
    score = torch.rand(B, H, Lmax, generator=g) ** 4
    if dyadic:
        score = (score * 16).floor() / 16
    if flat:
        score = torch.full_like(score, 0.25)
    kind = torch.randint(0, 3, (B, H, Lmax), generator=g).to(torch.uint8)
    if image_only:
        kind[:] = 1
    kind[:, :, :protected] = 0
    pos = torch.arange(Lmax, dtype=torch.int32).repeat(B, H, 1).contiguous()
    length = torch.tensor(lens, dtype=torch.int32).view(B, H)
    return [k, v, score, kind, pos, length]


def _kv_case(ctx, dtype, B, H, Lmax, d, lens, seed, **kw):
    host = _cache(dtype, B, H, Lmax, d, lens, seed, dyadic=kw.pop("dyadic", False), flat=kw.pop("flat", False),
                  image_only=kw.pop("image_only", False), protected=kw.pop("protected", 4))
    dev = [t.to(DEV) for t in host]
    nev = ctx.kv_compress(*dev, **kw)
    okw = dict(mode="threshold" if kw["mode"] == lv.KV_THRESHOLD else "budget", beta=kw.get("beta", 0.995),
               budget=kw.get("budget", 0), n_recent=kw.get("n_recent", 0), order=kw.get("order", lv.ORDER_STABLE))
    ref = O.kv_compress(f64(host[0]), f64(host[1]), host[2].numpy(), host[3].numpy(), host[4].numpy(),
                        host[5].numpy(), **okw)
    new_len = dev[5].cpu().numpy()
    assert np.array_equal(new_len, ref[5])
    assert np.array_equal(nev.cpu().numpy(), ref[6])
    for b in range(B):
        for h in range(H):
            n = int(new_len[b, h])
            assert np.array_equal(f64(dev[0][b, h, :n]), ref[0][b, h, :n])      # moves are byte-exact
            assert np.array_equal(f64(dev[1][b, h, :n]), ref[1][b, h, :n])
            assert np.array_equal(dev[2][b, h, :n].cpu().numpy(), ref[2][b, h, :n])
            assert np.array_equal(dev[3][b, h, :n].cpu().numpy(), ref[3][b, h, :n])
            assert np.array_equal(dev[4][b, h, :n].cpu().numpy(), ref[4][b, h, :n])
    return new_len, host[5].numpy()


@pytest.mark.parametrize("order", [lv.ORDER_STABLE, lv.ORDER_FILL])
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_kv_compress_threshold(ctx, order, dtype, d):
    lens = [1500, 1, 0, 777, 1024, 2047]
    for beta in (0.5, 0.9, 0.995):
        new_len, old = _kv_case(ctx, dtype, 3, 2, 2048, d, lens, 20, mode=lv.KV_THRESHOLD, beta=beta, order=order)
        assert (new_len <= old).all() and new_len[0, 0] < 1500
    _kv_case(ctx, dtype, 3, 2, 2048, d, lens, 21, mode=lv.KV_THRESHOLD, beta=0.7, order=order, dyadic=True)  # ties
    new_len, old = _kv_case(ctx, dtype, 3, 2, 2048, d, lens, 22, mode=lv.KV_THRESHOLD, beta=1.0, order=order)
    assert np.array_equal(new_len, old)                                                          # identity


@pytest.mark.parametrize("order", [lv.ORDER_STABLE, lv.ORDER_FILL])
def test_kv_compress_budget(ctx, order):
    lens = [1025, 1024, 300, 2048, 1026, 5]
    for budget, n_recent in ((1024, 1), (256, 0), (3, 2), (1, 0)):
        new_len, old = _kv_case(ctx, torch.bfloat16, 3, 2, 2048, 128, lens, 30, mode=lv.KV_BUDGET, budget=budget,
                                n_recent=n_recent, order=order, dyadic=budget == 256)
        for o, n in zip(old.ravel(), new_len.ravel()):
            assert n == o if o <= budget else n >= budget
    new_len, old = _kv_case(ctx, torch.bfloat16, 3, 2, 2048, 128, lens, 31, mode=lv.KV_BUDGET, budget=4096,
                            order=order)
    assert np.array_equal(new_len, old)


def test_kv_compress_bulk_config5_head(ctx):
    # one layer of config 5 after prefill: 8 heads x 16512 entries down to the 2048 budget, STABLE
    L = 16512
    new_len, _ = _kv_case(ctx, torch.bfloat16, 1, 8, L, 128, [L] * 8, 40, mode=lv.KV_BUDGET, budget=2048,
                          n_recent=0, order=lv.ORDER_STABLE, image_only=True, protected=128)
    assert (new_len == 2048).all()
    # and the paper's rule on the same shape: beta = 0.995 of the image score mass per head
    new_len, _ = _kv_case(ctx, torch.bfloat16, 1, 8, L, 128, [L] * 8, 41, mode=lv.KV_THRESHOLD, beta=0.995,
                          order=lv.ORDER_STABLE, image_only=True, protected=128)
    assert (new_len < L).all() and (new_len > 128).all()


@pytest.mark.parametrize("order", [lv.ORDER_STABLE, lv.ORDER_FILL])
def test_kv_compress_every_length_class(ctx, order):
    # the selection kernel keeps keys in registers up to 2048 / 4096 / 8192 / 17408 slots per head and
    # re-reads them beyond that: one ragged case per class, both rules
    for Lmax, lens in ((3000, [2999, 2500]), (6000, [5999, 4097]), (12000, [11111, 8193]), (20000, [19990, 17409])):
        _kv_case(ctx, torch.bfloat16, 1, 2, Lmax, 64, lens, 42 + Lmax, mode=lv.KV_BUDGET, budget=Lmax // 2, n_recent=2,
                 order=order)
        _kv_case(ctx, torch.bfloat16, 1, 2, Lmax, 64, lens, 43 + Lmax, mode=lv.KV_THRESHOLD, beta=0.9, order=order)
    # few distinct scores, and all candidates sharing one score (no bit of the keys differs)
    _kv_case(ctx, torch.bfloat16, 1, 2, 3000, 64, [2999, 2500], 44, mode=lv.KV_THRESHOLD, beta=0.6, order=order, dyadic=True)
    _kv_case(ctx, torch.bfloat16, 1, 2, 3000, 64, [2999, 2500], 45, mode=lv.KV_THRESHOLD, beta=0.6, order=order, flat=True)
    _kv_case(ctx, torch.bfloat16, 1, 2, 3000, 64, [2999, 2500], 46, mode=lv.KV_BUDGET, budget=1700, order=order, flat=True)


@pytest.mark.parametrize("order", [lv.ORDER_STABLE, lv.ORDER_FILL])
def test_kv_compress_many_short_heads(ctx, order):
    # more than 512 short heads take workgroups of 256 threads with eight keys per thread: ragged lengths,
    # both rules, ties included
    B, H, Lmax = 36, 16, 1100
    g = torch.Generator().manual_seed(77)
    lens = torch.randint(0, Lmax + 1, (B * H,), generator=g).tolist()
    lens[:6] = [1100, 1099, 1, 0, 257, 1025]
    _kv_case(ctx, torch.bfloat16, B, H, Lmax, 64, lens, 78, mode=lv.KV_THRESHOLD, beta=0.9, order=order)
    _kv_case(ctx, torch.bfloat16, B, H, Lmax, 64, lens, 79, mode=lv.KV_BUDGET, budget=400, n_recent=3, order=order,
             dyadic=True)


@pytest.mark.parametrize("order", [lv.ORDER_STABLE, lv.ORDER_FILL])
def test_kv_compress_special_scores(ctx, order):
    # NaN, negative, infinite, zero and tied scores: NaN ranks lowest and weighs nothing, negatives weigh
    # nothing, +inf is clamped to 2^16 in the mass; both rules must still agree with the oracle bit for bit
    B, H, Lmax, d = 1, 3, 700, 64
    host = _cache(torch.bfloat16, B, H, Lmax, d, [700, 650, 333], 120)
    g = torch.Generator().manual_seed(121)
    sc = host[2]
    pick = torch.randint(0, 8, sc.shape, generator=g)
    sc[pick == 0] = float("nan")
    sc[pick == 1] = -1.5
    sc[pick == 2] = 0.0
    sc[pick == 3] = -0.0
    sc[pick == 4] = 0.125
    sc[0, 1, 5] = float("inf")
    sc[0, 2, 7] = float("-inf")
    sc[0, 0, 9] = 3.0e5
    for kw in (dict(mode=lv.KV_BUDGET, budget=400, n_recent=3), dict(mode=lv.KV_BUDGET, budget=300, n_recent=0),
               dict(mode=lv.KV_THRESHOLD, beta=0.9), dict(mode=lv.KV_THRESHOLD, beta=0.5)):
        dev = [t.clone().to(DEV) for t in host]
        nev = ctx.kv_compress(*dev, order=order, **kw)
        okw = dict(mode="threshold" if kw["mode"] == lv.KV_THRESHOLD else "budget", beta=kw.get("beta", 0.995),
                   budget=kw.get("budget", 0), n_recent=kw.get("n_recent", 0), order=order)
        ref = O.kv_compress(f64(host[0]), f64(host[1]), host[2].numpy(), host[3].numpy(), host[4].numpy(),
                            host[5].numpy(), **okw)
        new_len = dev[5].cpu().numpy()
        assert np.array_equal(new_len, ref[5]), kw
        assert np.array_equal(nev.cpu().numpy(), ref[6])
        for h in range(H):
            n = int(new_len[0, h])
            assert np.array_equal(dev[4][0, h, :n].cpu().numpy(), ref[4][0, h, :n]), (kw, h)      # which entries, in order
            assert np.array_equal(dev[3][0, h, :n].cpu().numpy(), ref[3][0, h, :n])
            assert np.array_equal(f64(dev[0][0, h, :n]), ref[0][0, h, :n])
            got, want = dev[2][0, h, :n].cpu().numpy(), ref[2][0, h, :n]
            assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])


def test_one_threshold_keeps_fewer_entries_the_deeper_the_layer(ctx):
    """Sec. 3.2.2: one threshold beta for every layer keeps many entries where attention is spread out (shallow
    layers) and few where it is concentrated (deep layers; Sec. 3.1, Fig. 2b).  Pilot-study shape (1476 image tokens
    at every layer, concentration growing with depth): GPU scores, GPU compression at the paper's beta = 0.995, the
    oracle deciding on the GPU's score bits -- kept sets identical, kept counts falling with depth in every head."""
    w = configs.CFG7
    N, H, d, img0 = w.seq_len, w.n_kv_heads, w.head_dim, w.n_sys
    kept = []
    for layer in (1, 9, 18, 27):
        x = synth.layer_inputs(w, layer=layer)
        Lmax = N + 8
        kc = torch.zeros(1, H, Lmax, d, dtype=torch.bfloat16, device=DEV)
        vc = torch.zeros_like(kc)
        kc[:, :, :N] = x["k"].to(DEV).permute(0, 2, 1, 3)
        vc[:, :, :N] = x["v"].to(DEV).permute(0, 2, 1, 3)
        score = torch.zeros(1, H, Lmax, device=DEV)
        ctx.score_tokens(x["q"].to(DEV), x["k"].to(DEV), q_pos0=img0 + w.n_img, img_begin=img0, n_img=w.n_img,
                         score_head=score[:, :, img0:img0 + w.n_img])
        osh, _ = O.score_tokens(f64(x["q"]), f64(x["k"]), q_pos0=img0 + w.n_img, img_begin=img0, n_img=w.n_img)
        assert rel_err(score[:, :, img0:img0 + w.n_img].cpu(), osh) < 1e-5
        kind = torch.zeros(1, H, Lmax, dtype=torch.uint8, device=DEV)
        kind[:, :, img0:img0 + w.n_img] = lv.KIND_IMAGE
        pos = torch.arange(Lmax, dtype=torch.int32, device=DEV).view(1, 1, Lmax).expand(1, H, Lmax).contiguous()
        length = torch.full((1, H), N, dtype=torch.int32, device=DEV)
        state = [kc, vc, score, kind, pos, length]
        before = [f64(kc), f64(vc), score.cpu().numpy().copy(), kind.cpu().numpy(), pos.cpu().numpy(), length.cpu().numpy()]
        ctx.kv_compress(*state, mode=lv.KV_THRESHOLD, beta=w.kv_beta, order=lv.ORDER_STABLE, len_bound=N)
        ref = O.kv_compress(*before, mode="threshold", beta=w.kv_beta, order=O.ORDER_STABLE)
        new_len = length.cpu().numpy()
        assert np.array_equal(new_len, ref[5])
        for h in range(H):
            n = int(new_len[0, h])
            assert np.array_equal(pos[0, h, :n].cpu().numpy(), ref[4][0, h, :n])          # the same entries, in order
            assert np.array_equal(f64(kc[0, h, :n]), ref[0][0, h, :n])
        kept.append(new_len[0] - (w.n_sys + w.n_text))                                    # image entries kept per head
    kept = np.stack(kept)
    assert (kept[:-1] > kept[1:]).all(), kept
    assert kept[0].min() > 1.15 * kept[-1].max()


# --------------------------------------------------------------------------- step 6
def _attn_case(ctx, dtype, B, Hq, Hkv, d, Lmax, lens, seed, append=True, decay=0.9, track=True, len_bound=0):
    host = _cache(dtype, B, Hkv, Lmax, d, lens, seed)
    q = _rand((B, Hq, d), dtype, seed + 5)
    kn = _rand((B, Hkv, d), dtype, seed + 6) if append else None
    vn = _rand((B, Hkv, d), dtype, seed + 7) if append else None
    dev = [t.to(DEV) for t in host]
    out = ctx.decode_attn(q.to(DEV), None if kn is None else kn.to(DEV), None if vn is None else vn.to(DEV),
                          dev[0], dev[1], dev[2] if track else None, dev[3], dev[4], dev[5], score_decay=decay,
                          new_pos=4242, len_bound=len_bound)
    ref = O.decode_attn(f64(q), None if kn is None else f64(kn), None if vn is None else f64(vn), f64(host[0]),
                        f64(host[1]), host[2].numpy(), host[3].numpy(), host[4].numpy(), host[5].numpy(),
                        score_decay=decay, new_pos=4242, out_dtype="bf16" if dtype == torch.bfloat16 else "f32",
                        update_score=track)
    assert rel_err(f64(out.cpu()), ref[0]) < TOL[dtype]
    new_len = dev[5].cpu().numpy()
    assert np.array_equal(new_len, ref[6])
    for b in range(B):
        for h in range(Hkv):
            n = int(new_len[b, h])
            assert np.array_equal(f64(dev[0][b, h, :n]), ref[1][b, h, :n])
            assert np.array_equal(f64(dev[1][b, h, :n]), ref[2][b, h, :n])
            assert np.array_equal(dev[3][b, h, :n].cpu().numpy(), ref[4][b, h, :n])
            assert np.array_equal(dev[4][b, h, :n].cpu().numpy(), ref[5][b, h, :n])
            if track and n:
                assert rel_err(dev[2][b, h, :n].cpu().numpy(), ref[3][b, h, :n]) < 1e-5
            elif n:
                assert np.array_equal(dev[2][b, h, :n - int(append)].cpu().numpy(), ref[3][b, h, :n - int(append)])


def test_decode_attn_shapes(ctx):
    _attn_case(ctx, torch.bfloat16, 2, 14, 2, 128, 1100, [1024, 37, 0, 700], 50)                 # G=7, ragged, empty head
    _attn_case(ctx, torch.bfloat16, 2, 12, 2, 128, 600, [511, 512, 513, 1], 51, decay=1.0)       # G=6
    _attn_case(ctx, torch.float32, 1, 4, 4, 64, 360, [352, 100, 129, 128], 52)                   # config 1 shape, G=1
    _attn_case(ctx, torch.bfloat16, 1, 8, 2, 64, 300, [299, 150], 53)                            # d=64, G=4
    _attn_case(ctx, torch.float32, 1, 4, 2, 128, 200, [33, 199], 54)                             # fp32 d=128, G=2
    _attn_case(ctx, torch.bfloat16, 2, 14, 2, 128, 1100, [1024, 37, 5, 700], 55, append=False)   # no append
    _attn_case(ctx, torch.bfloat16, 2, 14, 2, 128, 1100, [1024, 37, 5, 700], 56, track=False)    # no importance
    _attn_case(ctx, torch.bfloat16, 2, 14, 2, 128, 4096, [1024, 37, 5, 700], 57, len_bound=1025)  # bound < Lmax
    _attn_case(ctx, torch.bfloat16, 1, 14, 2, 128, 9100, [9000, 8193], 58)                       # long cache: separate fold
    for seed in (59, 60, 61):                                                                    # same shape, same workspace,
        _attn_case(ctx, torch.bfloat16, 2, 14, 2, 128, 1100, [1024, 37, 0, 700], seed)           # again and again


def test_decode_attn_heads_at_or_beyond_the_length_bound(ctx):
    """The lengths live on the device, so a head can break the caller's len_bound promise without the host seeing
    it (the fused eviction may find nothing to evict).  Such a head must be handled inside the bound: a full
    head (len == bound) drops the new entry and attends to what it holds; a head longer than the bound attends to
    its first `bound` entries; neither has its length, its cache or anything beyond the bound touched.  Heads that
    keep the promise are unaffected.  Checked for the one-tile and several-tile forms, fp32, and with eviction."""
    for dtype, d, Hq, Hkv, Lmax, bound, lens, budget in (
            (torch.bfloat16, 128, 14, 2, 1100, 1025, [1025, 1040, 1024, 600], 0),      # 8 splits + the extra tile
            (torch.bfloat16, 128, 14, 2, 1100, 1025, [1025, 1040, 1024, 600], 1024),   # ... with the fused eviction
            (torch.bfloat16, 64, 8, 2, 700, 640, [640, 699, 639, 1], 0),               # whole 128-entry splits
            (torch.float32, 64, 4, 4, 400, 300, [300, 350, 299, 17, 300, 301, 0, 128], 0),
            (torch.bfloat16, 128, 4, 2, 5000, 4100, [4100, 4999, 4099, 2047], 4099)):  # long splits, eviction
        B = len(lens) // Hkv
        host = _cache(dtype, B, Hkv, Lmax, d, lens, 140)
        q, kn, vn = _rand((B, Hq, d), dtype, 141), _rand((B, Hkv, d), dtype, 142), _rand((B, Hkv, d), dtype, 143)
        dev = [t.to(DEV) for t in host]
        out = ctx.decode_attn(q.to(DEV), kn.to(DEV), vn.to(DEV), *dev, score_decay=0.9, new_pos=9, len_bound=bound,
                              evict_budget=budget, evict_recent=1)
        got = [t.cpu() for t in dev]
        G = Hq // Hkv
        for b in range(B):
            for h in range(Hkv):
                n0 = lens[b * Hkv + h]
                one = [f64(host[0][b:b + 1, h:h + 1]), f64(host[1][b:b + 1, h:h + 1]), host[2][b:b + 1, h:h + 1].numpy(),
                       host[3][b:b + 1, h:h + 1].numpy(), host[4][b:b + 1, h:h + 1].numpy(),
                       np.array([[min(n0, bound)]], dtype=np.int32)]
                fits = n0 < bound
                ref = O.decode_attn(f64(q[b:b + 1, h * G:(h + 1) * G]), f64(kn[b:b + 1, h:h + 1]) if fits else None,
                                    f64(vn[b:b + 1, h:h + 1]) if fits else None, *one, score_decay=0.9, new_pos=9,
                                    out_dtype="bf16" if dtype == torch.bfloat16 else "f32")
                assert rel_err(f64(out[b, h * G:(h + 1) * G].cpu()), ref[0][0]) < TOL[dtype], (b, h)
                n_att = int(ref[6][0, 0])
                state = list(ref[1:])
                if budget and n_att > budget and n0 <= bound:
                    mid = [state[0], state[1], got[2][b:b + 1, h:h + 1].numpy().copy(), state[3], state[4], state[5]]
                    # (the eviction is decided on the GPU's updated score bits; a slot already moved holds its
                    # mover's score, so take the scores from a second, eviction-free call below)
                    plain = [t.to(DEV) for t in host]
                    ctx.decode_attn(q.to(DEV), kn.to(DEV), vn.to(DEV), *plain, score_decay=0.9, new_pos=9, len_bound=bound)
                    mid[2] = plain[2][b:b + 1, h:h + 1].cpu().numpy()
                    state = list(O.kv_compress(*mid, mode="budget", budget=n_att - 1, n_recent=1, order=O.ORDER_FILL)[:6])
                    n_new = int(state[5][0, 0])
                    assert int(got[5][b, h]) == n_new
                    for i in (0, 1, 3, 4):
                        want = state[i][0, 0, :n_new]
                        have = got[i][b, h, :n_new]
                        assert np.array_equal(f64(have) if i < 2 else have.numpy(), want), (b, h, i)
                    assert np.array_equal(got[2][b, h, :n_new].numpy(), state[2][0, 0, :n_new])
                else:
                    # the length: grown by one where the entry fitted, else exactly what it was
                    assert int(got[5][b, h]) == (n0 + 1 if fits else n0), (b, h)
                    for i in (0, 1, 3, 4):
                        want = state[i][0, 0, :n_att]
                        have = got[i][b, h, :n_att]
                        assert np.array_equal(f64(have) if i < 2 else have.numpy(), want), (b, h, i)
                    if n_att:
                        assert rel_err(got[2][b, h, :n_att].numpy(), state[2][0, 0, :n_att]) < 1e-5
                # nothing at or beyond the attended entries was written (a dropped entry leaves no trace)
                for i in range(5):
                    assert torch.equal(got[i][b, h, n_att:], host[i][b, h, n_att:]), (b, h, i)


def _guarded(call):
    """Runs call(ctx, reserve) twice on fresh inputs: once to learn the scratch size the library asks for, once with
    a workspace of exactly that size in front of a guard band, which must come back untouched."""
    import ctypes as C
    from paper_2509_00419_amd import binding as bd
    probe = lv.Context(0)
    call(probe, True)
    torch.cuda.synchronize()
    need = 0 if probe._ws is None else probe._ws.numel()
    own = lv.Context(0)
    guard = 1 << 16
    ws = torch.full((need + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    own._ws = ws
    own._check(bd.lib.lvlm_set_workspace(own._h, C.c_void_p(ws.data_ptr()), need))
    call(own, False)
    torch.cuda.synchronize()
    assert bool((ws[need:] == 0xA5).all())


def test_no_call_writes_past_the_workspace_it_asked_for(ctx):
    # decode attention: heads at and beyond the bound, ragged short heads, every launch form
    for dtype, d, Hq, Hkv, Lmax, bound, lens, budget in (
            (torch.bfloat16, 128, 14, 2, 1100, 1025, [1025, 1040, 1024, 600], 1024),
            (torch.bfloat16, 64, 8, 2, 700, 640, [640, 699, 639, 1], 0),
            (torch.float32, 64, 4, 4, 400, 300, [300, 350, 299, 17, 300, 301, 0, 128], 0),
            (torch.bfloat16, 128, 4, 2, 5000, 4100, [4100, 4999, 4099, 2047], 4099),
            (torch.bfloat16, 128, 8, 1, 2100, 2049, [2049], 2048)):
        B = len(lens) // Hkv

        def decode(c, reserve):
            dev = [t.to(DEV) for t in _cache(dtype, B, Hkv, Lmax, d, lens, 160)]
            q, kn, vn = (_rand(sh, dtype, 161 + i).to(DEV) for i, sh in enumerate(((B, Hq, d), (B, Hkv, d), (B, Hkv, d))))
            c.decode_attn(q, kn, vn, *dev, score_decay=0.9, new_pos=9, len_bound=bound, evict_budget=budget, evict_recent=1,
                          reserve=reserve)
        _guarded(decode)
    # cache compression: both rules and orders, ragged heads, a head beyond the bound, the long-head form
    for Lmax, bound, lens, kw in ((2048, 0, [1500, 1, 0, 777, 1024, 2047], dict(mode=lv.KV_THRESHOLD, beta=0.9, order=lv.ORDER_FILL)),
                                  (3000, 2000, [2000, 2500, 1999, 2049, 5, 0], dict(mode=lv.KV_BUDGET, budget=700, n_recent=2, order=lv.ORDER_STABLE)),
                                  (12000, 0, [11111, 8193, 12000, 1, 4096, 9000], dict(mode=lv.KV_BUDGET, budget=5000, n_recent=0, order=lv.ORDER_FILL))):
        def compress(c, reserve):
            dev = [t.to(DEV) for t in _cache(torch.bfloat16, 3, 2, Lmax, 64, lens, 170)]
            c.kv_compress(*dev, len_bound=bound, reserve=reserve, **kw)
        _guarded(compress)
    # merge: counting ranks and sorted blocks; scoring: the three launch forms
    for n_img, n_keep, B in ((1333, 400, 3), (9000, 3000, 2)):
        def merge(c, reserve):
            hid = _rand((B, n_img + 12, 264), torch.bfloat16, 180).to(DEV)
            score = torch.rand(B, n_img, generator=torch.Generator().manual_seed(181)).to(DEV)
            c.merge_compact([hid], score, img_begin=5, n_img=n_img, n_keep=n_keep, reserve=reserve)
        _guarded(merge)
    # (two passes, a chunk per workgroup, shared tiles in one launch, shared tiles with the keys in runs)
    for B, N, T, n_img, Hq, Hkv, form in ((1, 5000, 64, 4800, 8, 2, 0), (1, 845, 64, 717, 8, 2, 1), (48, 986, 96, 890, 8, 2, 2),
                                          (4, 2200, 128, 2072, 48, 8, 3)):
        def score(c, reserve):
            q = _rand((B, T, Hq, 128), torch.bfloat16, 190).to(DEV)
            k = _rand((B, N, Hkv, 128), torch.bfloat16, 191).to(DEV)
            kw = dict(q_pos0=N - T, img_begin=N - T - n_img, n_img=n_img)
            assert c.score_plan(c.score_desc(q, k, **kw)) == form
            c.score_tokens(q, k, reserve=reserve, **kw)
        _guarded(score)


def test_stream_probe_reads_and_leaves_everything_as_it_is(ctx):
    # the diagnostic read-only pass: any size that is a multiple of 16 bytes, any workgroup count; it writes nothing
    for nbytes, n_wg in ((16, 1), (4096 + 16, 3), (1 << 20, 1), (33587200, 512), (8392704, 4096)):
        src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=DEV)
        keep = src.clone()
        sink = torch.zeros(4, dtype=torch.int32, device=DEV)
        ctx.stream_probe(src, n_wg, sink)
        torch.cuda.synchronize()
        assert torch.equal(src, keep) and int(sink.abs().sum()) == 0
    with pytest.raises(lv.LvlmError):
        ctx.stream_probe(torch.zeros(8, dtype=torch.uint8, device=DEV), 1, torch.zeros(1, dtype=torch.int32, device=DEV))


def test_kv_compress_leaves_heads_beyond_the_length_bound_alone(ctx):
    # a head longer than len_bound is not compressed at all (nothing evicted, nothing moved); the others are
    host = _cache(torch.bfloat16, 2, 2, 3000, 64, [2000, 2500, 1999, 2049], 150)
    for kw in (dict(mode=lv.KV_BUDGET, budget=1500, n_recent=1, order=lv.ORDER_FILL),
               dict(mode=lv.KV_THRESHOLD, beta=0.9, order=lv.ORDER_STABLE)):
        dev = [t.to(DEV) for t in host]
        nev = ctx.kv_compress(*dev, len_bound=2000, **kw).cpu().numpy()
        short = [t.clone() for t in host]
        okw = dict(mode="threshold" if kw["mode"] == lv.KV_THRESHOLD else "budget", beta=kw.get("beta", 0.995),
                   budget=kw.get("budget", 0), n_recent=kw.get("n_recent", 0), order=kw["order"])
        ref = O.kv_compress(f64(short[0]), f64(short[1]), short[2].numpy(), short[3].numpy(), short[4].numpy(),
                            short[5].numpy(), **okw)
        for b, h in ((0, 1), (1, 1)):                                  # 2500 and 2049 entries: beyond the bound
            assert nev[b, h] == 0 and int(dev[5][b, h]) == int(host[5][b, h])
            for i in range(5):
                assert torch.equal(dev[i][b, h].cpu(), host[i][b, h])
        for b, h in ((0, 0), (1, 0)):
            n = int(ref[5][b, h])
            assert int(dev[5][b, h]) == n and nev[b, h] == ref[6][b, h] and n < int(host[5][b, h])
            assert np.array_equal(dev[4][b, h, :n].cpu().numpy(), ref[4][b, h, :n])
            assert np.array_equal(f64(dev[0][b, h, :n]), ref[0][b, h, :n])


def test_decode_attn_config4_layer_step(ctx):
    # one layer-step of config 4 at its real shape: B=16, 28/4 heads, 1024 entries + the new one
    w = configs.CFG4
    _attn_case(ctx, torch.bfloat16, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, 1056,
               [1024] * (w.batch * w.n_kv_heads), 60, len_bound=1025)


def _attn_evict_case(ctx, dtype, B, Hq, Hkv, d, Lmax, lens, budget, n_recent, seed, protected=4):
    """decode_attn with evict_budget must equal decode_attn followed, for every head now longer than the budget,
    by the oracle's budget eviction of exactly one entry (budget = length - 1, FILL order) decided on the GPU's
    updated score bits."""
    host = _cache(dtype, B, Hkv, Lmax, d, lens, seed, protected=protected)
    q, kn, vn = _rand((B, Hq, d), dtype, seed + 5), _rand((B, Hkv, d), dtype, seed + 6), _rand((B, Hkv, d), dtype, seed + 7)
    plain = [t.to(DEV) for t in host]
    fused = [t.to(DEV) for t in host]
    out_plain = ctx.decode_attn(q.to(DEV), kn.to(DEV), vn.to(DEV), *plain, score_decay=0.9, new_pos=77)
    out_fused = ctx.decode_attn(q.to(DEV), kn.to(DEV), vn.to(DEV), *fused, score_decay=0.9, new_pos=77,
                                evict_budget=budget, evict_recent=n_recent)
    assert torch.equal(out_plain, out_fused)
    mid = [t.cpu() for t in plain]
    got = [t.cpu() for t in fused]
    for b in range(B):
        for h in range(Hkv):
            n = int(mid[5][b, h])
            one = [f64(mid[0][b:b + 1, h:h + 1]), f64(mid[1][b:b + 1, h:h + 1]), mid[2][b:b + 1, h:h + 1].numpy(),
                   mid[3][b:b + 1, h:h + 1].numpy(), mid[4][b:b + 1, h:h + 1].numpy(), mid[5][b:b + 1, h:h + 1].numpy()]
            if n > budget:
                one = O.kv_compress(*one, mode="budget", budget=n - 1, n_recent=n_recent, order=O.ORDER_FILL)
            m = int(one[5][0, 0])
            assert int(got[5][b, h]) == m, (b, h, n, m)
            assert np.array_equal(f64(got[0][b, h, :m]), one[0][0, 0, :m])
            assert np.array_equal(f64(got[1][b, h, :m]), one[1][0, 0, :m])
            assert np.array_equal(got[2][b, h, :m].numpy(), one[2][0, 0, :m])
            assert np.array_equal(got[3][b, h, :m].numpy(), one[3][0, 0, :m])
            assert np.array_equal(got[4][b, h, :m].numpy(), one[4][0, 0, :m])
    return got[5].numpy()


def test_decode_attn_with_step_eviction(ctx):
    # heads at, one over, far over and under the budget; G = 7 and G = 1; fp32; a recent window
    new_len = _attn_evict_case(ctx, torch.bfloat16, 2, 14, 2, 128, 1100, [1024, 1023, 1060, 300], 1024, 1, 110)
    assert list(new_len.ravel()) == [1024, 1024, 1060, 301]
    _attn_evict_case(ctx, torch.float32, 1, 4, 4, 64, 300, [256, 257, 10, 255], 256, 4, 111)
    _attn_evict_case(ctx, torch.bfloat16, 1, 8, 2, 64, 5000, [4100, 2047], 2048, 0, 112)              # several chunks
    # every entry protected except the appended one, which the recent window shields: nothing can go
    new_len = _attn_evict_case(ctx, torch.bfloat16, 1, 2, 2, 128, 64, [40, 41], 8, 1, 113, protected=64)
    assert list(new_len.ravel()) == [41, 42]
    # config 4 at its real shape, three steps in a row on the same state
    w = configs.CFG4
    host = _cache(torch.bfloat16, w.batch, w.n_kv_heads, w.kv_budget + 8, w.head_dim, [w.kv_budget] * (w.batch * w.n_kv_heads),
                  114, protected=256, image_only=True)
    a_state = [t.to(DEV) for t in host]
    b_state = [t.to(DEV) for t in host]
    stream = synth.DecodeStream(w)
    for t in range(3):
        qt, kt, vt = (x.to(DEV) for x in stream.next())
        oa = ctx.decode_attn(qt, kt, vt, *a_state, score_decay=0.9, new_pos=1024 + t, len_bound=w.kv_budget + 1)
        ctx.kv_compress(*a_state, mode=lv.KV_BUDGET, budget=w.kv_budget, n_recent=1, order=lv.ORDER_FILL,
                        len_bound=w.kv_budget + 1)
        ob = ctx.decode_attn(qt, kt, vt, *b_state, score_decay=0.9, new_pos=1024 + t, len_bound=w.kv_budget + 1,
                             evict_budget=w.kv_budget, evict_recent=1)
        assert torch.equal(oa, ob)
        assert torch.equal(a_state[5], b_state[5]) and int(b_state[5].max()) == w.kv_budget
        n = w.kv_budget
        for x, y in zip(a_state[:5], b_state[:5]):
            assert torch.equal(x[:, :, :n], y[:, :, :n]), t


def test_identity_cases_leave_decode_output_bit_identical(ctx):
    host = _cache(torch.bfloat16, 2, 2, 512, 128, [500, 200, 333, 512], 70)
    q = _rand((2, 14, 128), torch.bfloat16, 71).to(DEV)
    dev = [t.to(DEV) for t in host]
    base = ctx.decode_attn(q, None, None, dev[0], dev[1], None, dev[3], dev[4], dev[5]).clone()
    ctx.kv_compress(*dev, mode=lv.KV_THRESHOLD, beta=1.0)
    ctx.kv_compress(*dev, mode=lv.KV_BUDGET, budget=512, n_recent=1, order=lv.ORDER_FILL)
    again = ctx.decode_attn(q, None, None, dev[0], dev[1], None, dev[3], dev[4], dev[5])
    assert torch.equal(base, again)
    for a, b in zip(dev, host):
        assert torch.equal(a.cpu(), b)


# --------------------------------------------------------------------------- config 1 end to end
def test_config1_full_pipeline_stepwise(ctx):
    """Score -> merge/compact (hidden, K, V, positions) -> cache -> 64 decode steps with
    per-step eviction.  Each GPU step is checked against the oracle run on the GPU's state
    just before that step, so one flipped near-tie cannot cascade."""
    w = configs.CFG1
    x = synth.layer_inputs(w)
    N, H, d = w.seq_len, w.n_kv_heads, w.head_dim
    n_keep = lv.schedule(w.n_img, 0.5, 1)[0]
    q, k = x["q"].to(DEV), x["k"].to(DEV)
    kw = dict(q_pos0=w.n_sys + w.n_img, img_begin=w.n_sys, n_img=w.n_img)
    sh, sm = ctx.score_tokens(q, k, **kw)
    osh, osm = O.score_tokens(f64(x["q"]), f64(x["k"]), **kw)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5
    planes = [x["hidden"], x["k"].view(1, N, -1), x["v"].view(1, N, -1), x["pos"], sh.cpu().permute(0, 2, 1).contiguous()]
    # the per-head scores ride along as a plane so that cache entries keep their importance
    pad = torch.zeros(1, N, H)
    pad[:, w.n_sys:w.n_sys + w.n_img] = planes[4]
    planes[4] = pad
    rules = [lv.RULE_WEIGHTED] * 3 + [lv.RULE_TOP, lv.RULE_WEIGHTED]
    outs, keep, merged = ctx.merge_compact([p.to(DEV) for p in planes], sm, img_begin=w.n_sys, n_img=w.n_img,
                                           n_keep=n_keep, rules=rules)
    oouts, okeep, omerged = O.merge_compact([f64(p) if p.dtype != torch.int32 else p.numpy() for p in planes],
                                            sm.cpu().numpy(), img_begin=w.n_sys, n_img=w.n_img, n_keep=n_keep,
                                            rules=rules, dtypes=["f32"] * 5)
    assert np.array_equal(keep.cpu().numpy(), okeep) and np.array_equal(merged.cpu().numpy(), omerged)
    for got, ref, p in zip(outs, oouts, planes):
        if p.dtype == torch.int32:
            assert np.array_equal(got.cpu().numpy(), ref)
        else:
            assert rel_err(f64(got.cpu()), ref) < 1e-5
    n_new = N - (w.n_img - n_keep)
    assert n_new == 32 + 288 + 32                                                  # schedule count

    # build the per-head cache from the compacted K/V planes
    Lmax = n_new + 8
    kc = torch.zeros(1, H, Lmax, d, device=DEV)
    vc = torch.zeros(1, H, Lmax, d, device=DEV)
    kc[:, :, :n_new] = outs[1].view(1, n_new, H, d).permute(0, 2, 1, 3)
    vc[:, :, :n_new] = outs[2].view(1, n_new, H, d).permute(0, 2, 1, 3)
    score = torch.zeros(1, H, Lmax, device=DEV)
    score[:, :, :n_new] = outs[4].permute(0, 2, 1)
    kind = torch.zeros(1, H, Lmax, dtype=torch.uint8, device=DEV)
    kind[:, :, w.n_sys:w.n_sys + n_keep] = 1
    pos = torch.zeros(1, H, Lmax, dtype=torch.int32, device=DEV)
    pos[:, :, :n_new] = outs[3].view(1, 1, n_new)
    length = torch.full((1, H), n_new, dtype=torch.int32, device=DEV)
    state = [kc, vc, score, kind, pos, length]

    def snapshot():
        s = [t.cpu() for t in state]
        return [f64(s[0]), f64(s[1]), s[2].numpy(), s[3].numpy(), s[4].numpy(), s[5].numpy()]

    def check_state(ref):
        now = snapshot()
        assert np.array_equal(now[5], ref[5])
        for h in range(H):
            n = int(now[5][0, h])
            for i in (0, 1, 3, 4):
                assert np.array_equal(now[i][0, h, :n], ref[i][0, h, :n])
            assert rel_err(now[2][0, h, :n], ref[2][0, h, :n]) < 1e-5

    # one-shot compression down to the budget, then 64 steps: append + attend, then evict one
    before = snapshot()
    ctx.kv_compress(*state, mode=lv.KV_BUDGET, budget=w.kv_budget, n_recent=1, order=lv.ORDER_STABLE)
    ref = O.kv_compress(*before, mode="budget", budget=w.kv_budget, n_recent=1, order=O.ORDER_STABLE)
    check_state(ref[:6])
    assert int(state[5].max()) == w.kv_budget
    stream = synth.DecodeStream(w)
    for t in range(w.decode_steps):
        qt, kt, vt = stream.next()
        before = snapshot()
        out = ctx.decode_attn(qt.to(DEV), kt.to(DEV), vt.to(DEV), *state, score_decay=0.9, new_pos=N + t,
                              len_bound=w.kv_budget + 1)
        ref = O.decode_attn(f64(qt), f64(kt), f64(vt), *before, score_decay=0.9, new_pos=N + t)
        assert rel_err(f64(out.cpu()), ref[0]) < 1e-5, t
        check_state(ref[1:])
        before = snapshot()
        ctx.kv_compress(*state, mode=lv.KV_BUDGET, budget=w.kv_budget, n_recent=1, order=lv.ORDER_FILL,
                        len_bound=w.kv_budget + 1)
        ref = O.kv_compress(*before, mode="budget", budget=w.kv_budget, n_recent=1, order=O.ORDER_FILL)
        check_state(ref[:6])
        assert int(state[5].min()) == w.kv_budget and int(state[5].max()) == w.kv_budget


# --------------------------------------------------------------------------- full-size cases of configs 3-5
def test_score_config5_full_size(ctx):
    # T=128, N=16512, 48/8 heads: 24 row chunks per key block, 256-key blocks, the largest score launch
    w = configs.CFG5
    q = _rand((1, w.n_text, w.n_q_heads, w.head_dim), torch.bfloat16, 80)
    k = _rand((1, w.seq_len, w.n_kv_heads, w.head_dim), torch.bfloat16, 81)
    kw = dict(q_pos0=w.n_sys + w.n_img, img_begin=w.n_sys, n_img=w.n_img)
    sh, sm = ctx.score_tokens(q.to(DEV), k.to(DEV), **kw)
    osh, osm = O.score_tokens(f64(q), f64(k), **kw)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5


def test_merge_compact_config5_first_stage(ctx):
    # 16384 -> 5091 image tokens of 6144 channels (two rank tiles, 11294 merged rows)
    w = configs.CFG5
    n_keep = lv.schedule(w.n_img, 0.03, 3)[0]
    assert n_keep == 5091
    _merge_case(ctx, torch.bfloat16, 1, w.n_sys, w.n_img, w.n_text, w.hidden, n_keep, extra_planes=False, seed=82)


def test_merge_compact_config3_first_stage(ctx):
    w = configs.CFG3
    n_keep = lv.schedule(w.n_img, 0.35, 3)[0]
    assert n_keep == 1263
    _merge_case(ctx, torch.bfloat16, w.batch, w.n_sys, w.n_img, w.n_text, w.hidden, n_keep, seed=83)


def test_config4_decode_steps_stepwise(ctx):
    """Config 4 shape (B=16, 28/4 heads, budget 1024): 6 decode steps with eviction every step, each GPU
    call checked against the oracle applied to the GPU state just before it."""
    w = configs.CFG4
    B, H, d = w.batch, w.n_kv_heads, w.head_dim
    host = _cache(torch.bfloat16, B, H, w.kv_budget + 8, d, [w.kv_budget] * (B * H), 84, protected=256, image_only=True)
    state = [t.to(DEV) for t in host]
    stream = synth.DecodeStream(w)

    def snapshot():
        s = [t.cpu() for t in state]
        return [f64(s[0]), f64(s[1]), s[2].numpy(), s[3].numpy(), s[4].numpy(), s[5].numpy()]

    for t in range(6):
        qt, kt, vt = stream.next()
        before = snapshot()
        out = ctx.decode_attn(qt.to(DEV), kt.to(DEV), vt.to(DEV), *state, score_decay=0.9, new_pos=1024 + t,
                              len_bound=w.kv_budget + 1)
        ref = O.decode_attn(f64(qt), f64(kt), f64(vt), *before, score_decay=0.9, new_pos=1024 + t, out_dtype="bf16")
        assert rel_err(f64(out.cpu()), ref[0]) < 2e-2, t
        now = snapshot()
        assert np.array_equal(now[5], ref[6])
        assert rel_err(now[2][:, :, :w.kv_budget + 1], ref[3][:, :, :w.kv_budget + 1]) < 1e-5
        before = now
        ctx.kv_compress(*state, mode=lv.KV_BUDGET, budget=w.kv_budget, n_recent=1, order=lv.ORDER_FILL,
                        len_bound=w.kv_budget + 1)
        ref = O.kv_compress(*before, mode="budget", budget=w.kv_budget, n_recent=1, order=O.ORDER_FILL)
        now = snapshot()
        assert np.array_equal(now[5], ref[5]) and int(now[5].min()) == w.kv_budget
        n = w.kv_budget
        for i in (0, 1, 2, 3, 4):
            assert np.array_equal(now[i][:, :, :n], ref[i][:, :, :n]), (t, i)


def test_degenerate_sizes(ctx):
    # one image token, one query row, one key; a cache with a single entry; nothing to keep but the merged slot
    q, k = _rand((1, 1, 2, 64), torch.float32, 90), _rand((1, 1, 2, 64), torch.float32, 91)
    sh, sm = ctx.score_tokens(q.to(DEV), k.to(DEV), q_pos0=0, img_begin=0, n_img=1)
    assert torch.allclose(sh.cpu(), torch.ones(1, 2, 1)) and torch.allclose(sm.cpu(), torch.ones(1, 1))
    _merge_case(ctx, torch.float32, 1, 0, 1, 0, 4, 1, extra_planes=False, seed=92)       # n_img = n_keep = 1
    _merge_case(ctx, torch.float32, 1, 0, 2, 0, 4, 1, extra_planes=False, seed=93)       # two tokens into one
    _merge_case(ctx, torch.bfloat16, 2, 1, 3, 1, 8, 2, seed=94)
    _attn_case(ctx, torch.bfloat16, 1, 2, 2, 128, 4, [0, 0], 95)                          # empty caches + append
    _attn_case(ctx, torch.bfloat16, 1, 2, 2, 128, 4, [1, 3], 96, append=False)
    _kv_case(ctx, torch.bfloat16, 1, 2, 8, 128, [0, 1], 97, mode=lv.KV_THRESHOLD, beta=0.5)
    _kv_case(ctx, torch.bfloat16, 1, 2, 8, 128, [8, 1], 98, mode=lv.KV_BUDGET, budget=1, n_recent=0, order=lv.ORDER_FILL)


# --------------------------------------------------------------------------- step 3b: similarity merge
def _similar_case(ctx, dtype, B, n_sys, n_img, n_txt, C, n_keep, seed, clusters=0, with_size=True, extra=True,
                  identical=False):
    """GPU dominant set must equal the oracle's; each GPU assignment must be an arg-max of the oracle's
    fp64 cosines up to 1e-5 (exactly the oracle's choice wherever its margin is larger than that); merged
    values are checked against the oracle's merge under the GPU's assignment."""
    N = n_sys + n_img + n_txt
    g = torch.Generator().manual_seed(seed)
    hid = torch.randn(B, N, C, generator=g)
    if clusters:
        centres = torch.randn(B, clusters, C, generator=g)
        which = torch.randint(0, clusters, (B, n_img), generator=g)
        hid[:, n_sys:n_sys + n_img] = torch.gather(centres, 1, which[:, :, None].expand(B, n_img, C)) + \
            0.1 * torch.randn(B, n_img, C, generator=g)
    if identical:
        hid[:, n_sys:n_sys + n_img] = hid[:, n_sys:n_sys + 1]
    hid = hid.to(dtype)
    score = torch.rand(B, n_img, generator=g)
    size = torch.randint(1, 4, (B, n_img), generator=g).float() if with_size else None
    planes, rules, dts = [hid], [lv.RULE_WEIGHTED], ["bf16" if dtype == torch.bfloat16 else "f32"]
    if extra:
        planes += [_rand((B, N, 24), dtype, seed + 1), torch.arange(B * N, dtype=torch.int32).view(B, N, 1)]
        rules += [lv.RULE_WEIGHTED, lv.RULE_TOP]
        dts += [dts[0], "f32"]
    outs, keep, assign, size_out = ctx.merge_similar([p.to(DEV) for p in planes], score.to(DEV), img_begin=n_sys,
                                                     n_img=n_img, n_keep=n_keep, rules=rules,
                                                     size=None if size is None else size.to(DEV))
    keep, assign = keep.cpu().numpy(), assign.cpu().numpy()
    np_planes = [f64(p) if p.dtype != torch.int32 else p.numpy() for p in planes]
    for b in range(B):
        dom, oassign, cos, rest = O.similarity_assign(np_planes[0][b, n_sys:n_sys + n_img], score[b].numpy(), n_keep)
        assert np.array_equal(keep[b], dom)
        assert np.array_equal(assign[b, dom], np.arange(n_keep))
        if rest.size:
            best = cos.max(axis=1)
            chosen = cos[np.arange(rest.size), assign[b, rest]]
            assert (chosen >= best - 1e-5).all()
            second = np.sort(cos, axis=1)[:, -2] if n_keep > 1 else np.full(rest.size, -np.inf)
            clear = best - second > 1e-5
            assert np.array_equal(assign[b, rest][clear], oassign[rest][clear])
            if identical:
                assert (assign[b, rest] == 0).all()                    # all cosines equal: lowest position wins
    oouts, _, _, onew = O.merge_similar(np_planes, score.numpy(), img_begin=n_sys, n_img=n_img, n_keep=n_keep,
                                        size=None if size is None else size.numpy(), rules=rules, dtypes=dts,
                                        assign=assign)
    np.testing.assert_allclose(size_out.cpu().numpy(), onew, rtol=1e-6)
    for got, ref, p in zip(outs, oouts, planes):
        assert tuple(got.shape) == ref.shape
        if p.dtype == torch.int32:
            assert np.array_equal(got.cpu().numpy(), ref)
        else:
            got = f64(got.cpu())
            assert np.array_equal(got[:, :n_sys], ref[:, :n_sys]) and np.array_equal(got[:, n_sys + n_keep:], ref[:, n_sys + n_keep:])
            assert rel_err(got, ref) < TOL[dtype]


def test_merge_similar(ctx):
    _similar_case(ctx, torch.float32, 1, 32, 576, 32, 256, 288, 100, clusters=16)               # config 1 shape
    _similar_case(ctx, torch.bfloat16, 1, 64, 2048, 64, 3584, 636, 101, clusters=64, extra=False)  # config 2 stage
    _similar_case(ctx, torch.bfloat16, 2, 3, 333, 5, 160, 77, 102, clusters=8)                   # ragged tiles, batch
    _similar_case(ctx, torch.bfloat16, 2, 3, 333, 5, 160, 77, 103, with_size=False)              # unclustered, unit sizes
    _similar_case(ctx, torch.float32, 1, 0, 300, 0, 64, 1, 104)                                  # one dominant token
    _similar_case(ctx, torch.float32, 1, 2, 200, 2, 64, 200, 105)                                # nothing removed
    _similar_case(ctx, torch.bfloat16, 1, 1, 500, 1, 128, 130, 106, identical=True)              # all ties
    _similar_case(ctx, torch.bfloat16, 1, 2, 150, 2, 72, 40, 107, clusters=4)                    # 144-byte rows: partial slice
    _similar_case(ctx, torch.bfloat16, 1, 2, 4500, 2, 64, 1200, 108, clusters=16)               # ranks by sorted blocks


# --------------------------------------------------------------------------- seeded random shapes, every entry point
def _random_lens(rng, n, Lmax, lo=0):
    edges = [127, 128, 129, 159, 160, 161, 255, 256, 257, 1023, 1024, 1025]
    out = []
    for _ in range(n):
        r = rng.random()
        if r < 0.1:
            out.append(lo)
        elif r < 0.2:
            out.append(Lmax - 1)
        elif r < 0.4:
            out.append(min(Lmax - 1, rng.choice(edges)))
        else:
            out.append(rng.randint(lo, Lmax - 1))
    return out


@pytest.mark.parametrize("seed", [1, 2])
def test_random_shapes_every_entry_point(ctx, seed):
    """Shapes drawn at random inside the documented limits (group sizes 1-8, both head sizes and dtypes, ragged and
    empty heads, lengths around the tile edges), each checked like the hand-picked cases above."""
    import random
    rng = random.Random(seed)
    combos = [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64), (torch.float32, 128)]

    def heads():
        hkv = rng.choice([1, 2, 3, 4, 8])
        return hkv * rng.randint(1, 8), hkv

    for _ in range(40):
        # score
        (dtype, d), (Hq, Hkv) = rng.choice(combos), heads()
        n_img = rng.choice([1, 2, 31, 33, 200, 717, rng.randint(1, 2600)])
        if dtype == torch.float32:
            n_img = min(n_img, 900)
        test_score_tokens(ctx, dtype, rng.randint(1, 3), rng.choice([1, 5, 31, 32, 33, 64, 96, rng.randint(1, 100)]), Hq,
                          Hkv, d, rng.choice([0, 3, 64, rng.randint(0, 70)]), n_img, rng.random() < 0.8)
        # merge
        n_img = rng.choice([1, 2, 3, 64, 65, 576, rng.randint(1, 3000)])
        _merge_case(ctx, rng.choice([torch.bfloat16, torch.float32]), rng.randint(1, 3), rng.randint(0, 9), n_img,
                    rng.randint(0, 9), rng.choice([1, 7, 64, 100, 256, 257, 520, 1024, rng.randint(1, 1200)]),
                    rng.choice([1, n_img, max(1, n_img - 1), rng.randint(1, n_img)]),
                    w_mode=rng.choice([None, None, lv.MERGE_PAIRWISE, lv.MERGE_LINEAR_RAW]),
                    extra_planes=rng.random() < 0.5, seed=rng.randint(0, 10000))
        # cache compression
        (dtype, d), B, H = rng.choice(combos), rng.randint(1, 2), rng.randint(1, 3)
        Lmax = rng.choice([8, 65, 700, 2048, 2049, 4100, rng.randint(5, 9000)])
        order = rng.choice([lv.ORDER_STABLE, lv.ORDER_FILL])
        if rng.random() < 0.5:
            kw = dict(mode=lv.KV_THRESHOLD, beta=rng.choice([0.3, 0.9, 0.995, 0.9999, 1.0]), order=order)
        else:
            kw = dict(mode=lv.KV_BUDGET, budget=rng.choice([1, 2, Lmax // 2 + 1, Lmax, rng.randint(1, Lmax)]),
                      n_recent=rng.choice([0, 1, 7]), order=order)
        _kv_case(ctx, dtype, B, H, Lmax, d, _random_lens(rng, B * H, Lmax + 1), rng.randint(0, 10000),
                 dyadic=rng.random() < 0.3, image_only=rng.random() < 0.3, protected=rng.choice([0, 4, min(Lmax, 64)]), **kw)
        # decode attention
        (dtype, d), (Hq, Hkv), B = rng.choice(combos), heads(), rng.randint(1, 3)
        Lmax = rng.choice([2, 33, 129, 161, 300, 1100, 2200, rng.randint(2, 5000)])
        append = rng.random() < 0.8
        lens = _random_lens(rng, B * Hkv, Lmax, lo=0 if append else 1)
        lb = 0
        if rng.random() < 0.4:
            lb = min(Lmax, max(lens) + int(append) + rng.choice([0, 1, 31, 200]))
        _attn_case(ctx, dtype, B, Hq, Hkv, d, Lmax, lens, rng.randint(0, 10000), append=append,
                   decay=rng.choice([0.9, 1.0, 0.0]), track=rng.random() < 0.8, len_bound=lb)
        # decode attention with the per-step eviction
        (dtype, d), (Hq, Hkv), B = rng.choice(combos), heads(), rng.randint(1, 2)
        Lmax = rng.choice([64, 300, 1100, 2500, rng.randint(16, 3000)])
        budget = rng.randint(1, Lmax - 1)
        lens = [min(Lmax - 1, max(0, budget + rng.choice([-5, -1, 0, 0, 1, 3, 40]))) for _ in range(B * Hkv)]
        _attn_evict_case(ctx, dtype, B, Hq, Hkv, d, Lmax, lens, budget, rng.choice([0, 1, 4]), rng.randint(0, 10000),
                         protected=rng.choice([0, 4]))
