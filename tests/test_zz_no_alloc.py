"""lvlm_decode_attn_static -- decode attention for callers that cannot allocate -- against lvlm_decode_attn.

Both entry points run the same kernels; the static one keeps their scratch (split partials, per-entry logits,
lengths) in a fixed array inside the library instead of the caller's workspace.  Every output of the static call
must equal the workspace call's bit for bit (attention rows, appended entries, updated importance, lengths, and
with evict_budget the evicted slots), on two calls in a row of which the second is smaller -- the array then still
holds the first call's partials and logits, which must not leak into the second result.
"""
import ctypes as C

import pytest
import torch

import paper_2509_00419_amd as lv
from paper_2509_00419_amd import binding as bd

DEV = "cuda:0"


def _state(dtype, B, Hkv, Lmax, d, lens, seed):
    g = torch.Generator().manual_seed(seed)
    k = torch.randn(B, Hkv, Lmax, d, generator=g).to(dtype)
    v = torch.randn(B, Hkv, Lmax, d, generator=g).to(dtype)
    score = torch.rand(B, Hkv, Lmax, generator=g) ** 4
    kind = torch.randint(0, 3, (B, Hkv, Lmax), generator=g).to(torch.uint8)
    kind[:, :, :4] = 0
    pos = torch.arange(Lmax, dtype=torch.int32).repeat(B, Hkv, 1).contiguous()
    length = torch.tensor(lens, dtype=torch.int32).view(B, Hkv)
    return [k, v, score, kind, pos, length]


def _both(ctx, dtype, B, Hq, Hkv, d, Lmax, lens, seed, **kw):
    host = _state(dtype, B, Hkv, Lmax, d, lens, seed)
    g = torch.Generator().manual_seed(seed + 1)
    q = torch.randn(B, Hq, d, generator=g).to(dtype).to(DEV)
    kn = torch.randn(B, Hkv, d, generator=g).to(dtype).to(DEV)
    vn = torch.randn(B, Hkv, d, generator=g).to(dtype).to(DEV)
    a = [t.to(DEV) for t in host]
    b = [t.to(DEV) for t in host]
    out_a = ctx.decode_attn(q, kn, vn, *a, score_decay=0.9, new_pos=5, **kw)
    out_b = ctx.decode_attn(q, kn, vn, *b, score_decay=0.9, new_pos=5, static_scratch=True, **kw)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b)
    assert torch.equal(a[5], b[5])
    for x, y, name in zip(a[:5], b[:5], ("k", "v", "score", "kind", "pos")):
        assert torch.equal(x, y), name
    assert not torch.equal(a[2].cpu(), host[2]) and bool(out_a.float().abs().sum() > 0)     # the call did something


@pytest.mark.gpu
def test_static_scratch_call_equals_the_workspace_call_twice_in_a_row():
    ctx = lv.Context(0)
    # first the config-4 layer-step shape with the fused eviction (4.2 MB of scratch), then a smaller, ragged one
    _both(ctx, torch.bfloat16, 16, 28, 4, 128, 1032, [1024] * 64, 200, len_bound=1025, evict_budget=1024, evict_recent=1)
    _both(ctx, torch.bfloat16, 2, 14, 2, 128, 700, [640, 37, 0, 300], 201)
    # and a third, fp32, smaller again, without a length bound
    _both(ctx, torch.float32, 1, 4, 4, 64, 300, [256, 257, 10, 255], 202, evict_budget=256, evict_recent=4)
    # a context that never had a workspace attached can make the static call
    fresh = lv.Context(0)
    host = _state(torch.bfloat16, 1, 2, 200, 128, [150, 7], 203)
    dev = [t.to(DEV) for t in host]
    q = torch.randn(1, 4, 128).bfloat16().to(DEV)
    out = fresh.decode_attn(q, None, None, *dev, static_scratch=True)
    ref = ctx.decode_attn(q, None, None, *[t.to(DEV) for t in host])
    torch.cuda.synchronize()
    assert fresh._ws is None and torch.equal(out, ref)


def test_static_scratch_call_refuses_shapes_beyond_its_array():
    # host-side check, before anything touches a GPU: 4096 sequences need far more than the 8 MiB array
    ctx = lv.Context(0)
    ad = bd.AttnDesc(bd.BF16, 4096, 28, 4, 128, 1056, 1025, 2, 0, 0.088, 0.9, 0, 0)
    st = bd.lib.lvlm_decode_attn_static(ctx._h, None, C.byref(ad), 256, None, None, 512, 768, None, None, None, 1024, 2048)
    assert st == 3 and b"built-in array" in bd.lib.lvlm_last_error(ctx._h)
    # argument errors come first, as in lvlm_decode_attn
    st = bd.lib.lvlm_decode_attn_static(ctx._h, None, C.byref(ad), None, None, None, 512, 768, None, None, None, 1024, 2048)
    assert st == 1
