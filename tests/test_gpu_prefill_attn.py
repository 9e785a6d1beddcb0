"""GPU parity of lvlm_prefill_attn (the layer's attention with the scores as its by-product) against the CPU
oracle, through the C ABI.

Tolerances (max |gpu - oracle| / max |oracle|): outputs 2e-2 (bf16) / 1e-5 (fp32); the row normalisers and
the scores are fp32 whatever the input dtype: 1e-5.
"""
import numpy as np
import pytest
import torch

import paper_2509_00419_amd as lv
from oracle import lvlm_oracle as O
from workloads import configs

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


def _qkv(B, N, Hq, Hkv, d, dtype, seed, q_gain=1.0):
    """q, k, v as views of one fused projection output [B, N, Hq + 2 Hkv, d], as a model lays them out."""
    g = torch.Generator().manual_seed(seed)
    fused = torch.randn(B, N, Hq + 2 * Hkv, d, generator=g)
    fused[:, :, :Hq] *= q_gain
    fused = fused.to(dtype)
    return fused, (lambda t: (t[:, :, :Hq], t[:, :, Hq:Hq + Hkv], t[:, :, Hq + Hkv:]))


CASES = [
    # dtype, B, N, Hq, Hkv, d, causal, T, img_begin, n_img, q_gain        what it covers
    (torch.float32, 1, 640, 4, 4, 64, True, 32, 32, 576, 1.0),            # config 1
    (torch.float32, 2, 77, 4, 2, 128, True, 5, 3, 60, 2.0),               # fp32, d = 128, ragged
    (torch.float32, 1, 130, 2, 1, 64, False, 0, 0, 0, 1.0),               # fp32, no mask, attention only
    (torch.bfloat16, 2, 333, 6, 2, 128, True, 9, 5, 300, 1.0),            # ragged rows and keys, G = 3
    (torch.bfloat16, 1, 233, 8, 8, 64, False, 0, 0, 0, 1.0),              # d = 64, no mask, attention only
    (torch.bfloat16, 1, 257, 4, 2, 64, True, 40, 10, 200, 3.0),           # d = 64 causal, peaky rows, one row past a block
    (torch.bfloat16, 3, 500, 8, 4, 128, True, 64, 20, 400, 1.0),          # 12 (batch, KV head) pairs: 8 + 4 over the XCDs
    (torch.bfloat16, 1, 31, 2, 2, 128, True, 31, 0, 20, 1.0),             # shorter than one tile, every row an instruction row
    (torch.bfloat16, 1, 1, 2, 1, 128, True, 1, 0, 1, 1.0),                # one token
    (torch.float32, 1, 1, 2, 2, 64, True, 1, 0, 1, 1.0),                  # one token, fp32
    (torch.bfloat16, 2, 150, 4, 2, 128, False, 10, 5, 100, 1.0),          # scores without a causal mask
    (torch.bfloat16, 1, 128, 2, 1, 128, True, 3, 0, 125, 1.0),            # exactly one full query block
    (torch.bfloat16, 1, 2176, 28, 4, 128, True, 64, 64, 2048, 1.0),       # config 2 layer
]


@pytest.mark.parametrize("dtype,B,N,Hq,Hkv,d,causal,T,img0,n_img,gain", CASES)
def test_prefill_attn_matches_oracle(ctx, dtype, B, N, Hq, Hkv, d, causal, T, img0, n_img, gain):
    fused, split = _qkv(B, N, Hq, Hkv, d, dtype, 100 + N, gain)
    q, k, v = split(fused)
    qd, kd, vd = split(fused.to(DEV))
    out, lse, sh, sm = ctx.prefill_attn(qd, kd, vd, causal=causal, n_text=T, img_begin=img0, n_img=n_img)
    torch.cuda.synchronize()
    o_out, o_lse = O.prefill_attn(f64(q), f64(k), f64(v), causal=causal, dtype="bf16" if dtype == torch.bfloat16 else "f32")
    assert rel_err(out.float().cpu(), o_out) < TOL[dtype]
    assert np.abs(lse.cpu().numpy() - o_lse).max() < 1e-5 * max(1.0, np.abs(o_lse).max())
    if T > 0:
        osh, osm = O.score_tokens(f64(q[:, N - T:]), f64(k), q_pos0=N - T, img_begin=img0, n_img=n_img, causal=causal)
        assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5
        # and exactly what lvlm_score_tokens gives from the same normalisers
        sh2, sm2 = ctx.score_tokens(qd[:, N - T:], kd, q_pos0=N - T, img_begin=img0, n_img=n_img, causal=causal,
                                    row_lse=lse[:, :, N - T:].contiguous())
        assert torch.equal(sh, sh2) and torch.equal(sm, sm2)
    else:
        assert sh is None and sm is None


def test_prefill_attn_config3_shape_two_sequences(ctx):
    # InternVL2.5-8B-shaped layer (32 / 8 heads, 1792 image + 96 text tokens), two of the eight sequences for the oracle
    w = configs.CFG3
    B, N = 2, w.seq_len
    fused, split = _qkv(B, N, w.n_q_heads, w.n_kv_heads, w.head_dim, torch.bfloat16, 7)
    q, k, v = split(fused)
    qd, kd, vd = split(fused.to(DEV))
    out, lse, sh, sm = ctx.prefill_attn(qd, kd, vd, n_text=w.n_text, img_begin=w.n_sys, n_img=w.n_img)
    o_out, o_lse = O.prefill_attn(f64(q), f64(k), f64(v), dtype="bf16")
    assert rel_err(out.float().cpu(), o_out) < 2e-2
    assert np.abs(lse.cpu().numpy() - o_lse).max() < 1e-5 * np.abs(o_lse).max()
    osh, osm = O.score_tokens(f64(q[:, N - w.n_text:]), f64(k), q_pos0=N - w.n_text, img_begin=w.n_sys, n_img=w.n_img)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5


def test_prefill_attn_config5_shape_sampled_group(ctx):
    # 16512 tokens, 48 / 8 heads on the GPU; the oracle checks one KV group (its 6 query heads), every row
    w = configs.CFG5
    N, Hq, Hkv, d = w.seq_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    fused, split = _qkv(1, N, Hq, Hkv, d, torch.bfloat16, 11)
    q, k, v = split(fused)
    qd, kd, vd = split(fused.to(DEV))
    out, lse, sh, sm = ctx.prefill_attn(qd, kd, vd, n_text=w.n_text, img_begin=w.n_sys, n_img=w.n_img)
    torch.cuda.synchronize()
    g, G = Hkv - 1, Hq // Hkv
    heads = slice(g * G, (g + 1) * G)
    o_out, o_lse = O.prefill_attn(f64(q[:, :, heads]), f64(k[:, :, g:g + 1]), f64(v[:, :, g:g + 1]), dtype="bf16")
    assert rel_err(out[:, :, heads].float().cpu(), o_out) < 2e-2
    assert np.abs(lse[:, heads].cpu().numpy() - o_lse).max() < 1e-5 * np.abs(o_lse).max()
    osh, _ = O.score_tokens(f64(q[:, N - w.n_text:, heads]), f64(k[:, :, g:g + 1]), q_pos0=N - w.n_text,
                            img_begin=w.n_sys, n_img=w.n_img)
    assert rel_err(sh[:, g:g + 1].cpu(), osh) < 1e-5
    # properties that hold for every head: rows are convex combinations of the values they see
    vmax = vd.float().abs().amax()
    assert float(out.float().abs().amax()) <= float(vmax) * (1 + 2 ** -7)
    assert torch.isfinite(lse).all()


def test_prefill_attn_logits_far_above_the_first_tile(ctx):
    """Rows whose later logits exceed everything in the first 32 keys by far more than fp32 can hold as a
    probability ratio (natural-log distance 120): the kernel that fixes its reference at the first tile must
    give these workgroups to the one that follows the running maximum.  Also the reverse (a dominant first key)
    and ordinary rows in the same launch."""
    B, N, Hq, Hkv, d = 1, 420, 4, 2, 64
    g = torch.Generator().manual_seed(3)
    q = 0.05 * torch.randn(B, N, Hq, d, generator=g)
    k = 0.05 * torch.randn(B, N, Hkv, d, generator=g)
    v = torch.randn(B, N, Hkv, d, generator=g)
    q[:, :, 0:2, 0] = 22.0                       # heads 0, 1 (KV head 0): logit = 22 * k0 / 8
    k[:, :32, 0, 0] = -22.0                      # first tile: -60.5
    k[:, 32:, 0, 0] = 22.0                       # later keys: +60.5
    k[:, 200, 0, 0] = 30.0                       # and one at +82.5
    q[:, :, 2, 0] = 22.0                         # head 2 (KV head 1): a dominant first key, the rest far below
    k[:, 0, 1, 0] = 22.0
    k[:, 1:, 1, 0] = -22.0
    q, k, v = q.bfloat16(), k.bfloat16(), v.bfloat16()
    out, lse, sh, sm = ctx.prefill_attn(q.to(DEV), k.to(DEV), v.to(DEV), n_text=20, img_begin=8, n_img=380)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    o_out, o_lse = O.prefill_attn(f64(q), f64(k), f64(v), dtype="bf16")
    assert rel_err(out.float().cpu(), o_out) < 2e-2
    assert np.abs(lse.cpu().numpy() - o_lse).max() < 1e-5 * np.abs(o_lse).max()
    osh, osm = O.score_tokens(f64(q[:, N - 20:]), f64(k), q_pos0=N - 20, img_begin=8, n_img=380)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5


def test_prefill_attn_far_logits_in_the_middle_of_a_long_row(ctx):
    """One sequence of nine query blocks with few heads; logits that jump far above everything before them in the
    middle of the rows (natural-log distance 120 and more), so that only the workgroups whose rows reach those keys
    take the fallback kernel, the others the plain one, in the same launch."""
    B, N, Hq, Hkv, d = 1, 1100, 4, 2, 128
    g = torch.Generator().manual_seed(5)
    q = 0.05 * torch.randn(B, N, Hq, d, generator=g)
    k = 0.05 * torch.randn(B, N, Hkv, d, generator=g)
    v = torch.randn(B, N, Hkv, d, generator=g)
    q[:, :, 0:2, 0] = 26.0                       # heads 0, 1: logit = 26 * k0 / sqrt(128)
    k[:, :, 0, 0] = -26.0                        # -59.8 everywhere ...
    k[:, 300:330, 0, 0] = 26.0                   # ... but +59.8 on 30 keys inside a later part
    k[:, 700, 0, 0] = 30.0
    q, k, v = q.bfloat16(), k.bfloat16(), v.bfloat16()
    out, lse, sh, sm = ctx.prefill_attn(q.to(DEV), k.to(DEV), v.to(DEV), n_text=40, img_begin=16, n_img=1000)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    o_out, o_lse = O.prefill_attn(f64(q), f64(k), f64(v), dtype="bf16")
    assert rel_err(out.float().cpu(), o_out) < 2e-2
    assert np.abs(lse.cpu().numpy() - o_lse).max() < 1e-5 * np.abs(o_lse).max()
    osh, osm = O.score_tokens(f64(q[:, N - 40:]), f64(k), q_pos0=N - 40, img_begin=16, n_img=1000)
    assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5


def test_prefill_attn_random_shapes(ctx):
    """Seeded sweep over small shapes: lengths around the tile and block edges, head counts and groups (G = 1 ... 7),
    both head dimensions and dtypes, with and without the mask, any number of instruction rows, any image span,
    flat and peaky rows."""
    rng = np.random.default_rng(20250901)
    for it in range(24):
        dtype = torch.bfloat16 if rng.random() < 0.8 else torch.float32
        d = int(rng.choice([64, 128]))
        Hkv, G = int(rng.choice([1, 2, 3, 4, 8])), int(rng.choice([1, 2, 4, 5, 7]))
        Hq = Hkv * G
        B = int(rng.choice([1, 1, 2, 3, 9]))
        N = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 255, 256, 257, 300, 511, 513, 640]))
        if dtype == torch.float32:
            N = min(N, 300)
        if B * Hq * N * N > 4e7:
            B = 1
        causal = bool(rng.random() < 0.8)
        T = int(rng.integers(0, min(N, 70) + 1))
        n_img = int(rng.integers(1, N + 1)) if T > 0 else 0
        img0 = int(rng.integers(0, N - n_img + 1)) if T > 0 else 0
        fused, split = _qkv(B, N, Hq, Hkv, d, dtype, 3000 + it, float(rng.choice([1.0, 1.0, 3.0, 6.0])))
        q, k, v = split(fused)
        qd, kd, vd = split(fused.to(DEV))
        out, lse, sh, sm = ctx.prefill_attn(qd, kd, vd, causal=causal, n_text=T, img_begin=img0, n_img=n_img)
        torch.cuda.synchronize()
        case = (it, dtype, B, N, Hq, Hkv, d, causal, T, img0, n_img)
        o_out, o_lse = O.prefill_attn(f64(q), f64(k), f64(v), causal=causal, dtype="bf16" if dtype == torch.bfloat16 else "f32")
        assert rel_err(out.float().cpu(), o_out) < TOL[dtype], case
        assert np.abs(lse.cpu().numpy() - o_lse).max() < 1e-5 * max(1.0, np.abs(o_lse).max()), case
        if T > 0:
            osh, osm = O.score_tokens(f64(q[:, N - T:]), f64(k), q_pos0=N - T, img_begin=img0, n_img=n_img, causal=causal)
            assert rel_err(sh.cpu(), osh) < 1e-5 and rel_err(sm.cpu(), osm) < 1e-5, case


def test_prefill_attn_rejects_bad_arguments(ctx):
    fused, split = _qkv(1, 64, 4, 2, 64, torch.bfloat16, 1)
    qd, kd, vd = split(fused.to(DEV))
    with pytest.raises(lv.LvlmError):
        ctx.prefill_attn(qd, kd, vd, scale=0.0)                     # scale must be positive
    with pytest.raises(lv.LvlmError):
        ctx.prefill_attn(qd, kd, vd, n_text=65, img_begin=0, n_img=10)      # more instruction rows than rows
    with pytest.raises(lv.LvlmError):
        ctx.prefill_attn(qd, kd, vd, n_text=8, img_begin=60, n_img=10)      # image span outside the sequence
