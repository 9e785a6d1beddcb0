"""Pins for oracle.prefill_attn (the layer's own attention, whose row normalisers the scores of Sec. 3.2.1
are computed from).

Independent of the oracle's code: brute-force Python loops, a library attention routine in fp64, closed
forms, and the tie to the score oracle (its normaliser-free path must reproduce its own scores when fed
this function's normalisers).
"""
import math

import numpy as np
import torch

from oracle import lvlm_oracle as O


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _brute_force(q, k, v, scale, causal):
    B, N, Hq, d = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    out = np.zeros((B, N, Hq, d))
    lse = np.zeros((B, Hq, N))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for i in range(N):
                last = i if causal else N - 1
                logits = [scale * sum(float(q[b, i, h, c]) * float(k[b, j, g, c]) for c in range(d)) for j in range(last + 1)]
                mx = max(logits)
                den = sum(math.exp(x - mx) for x in logits)
                lse[b, h, i] = mx + math.log(den)
                for c in range(d):
                    out[b, i, h, c] = sum(math.exp(x - mx) / den * float(v[b, j, g, c]) for j, x in enumerate(logits))
    return out, lse


def test_brute_force_tiny_causal_and_full():
    q, k, v = _rand((2, 7, 4, 3), 1), _rand((2, 7, 2, 3), 2), _rand((2, 7, 2, 3), 3)
    for causal in (True, False):
        out, lse = O.prefill_attn(q, k, v, scale=0.7, causal=causal)
        bo, bl = _brute_force(q, k, v, 0.7, causal)
        np.testing.assert_allclose(out, bo, rtol=0, atol=2e-6)
        np.testing.assert_allclose(lse, bl, rtol=0, atol=2e-6)


def test_against_library_attention_fp64():
    B, N, Hq, Hkv, d = 2, 37, 6, 2, 16
    q, k, v = _rand((B, N, Hq, d), 4), _rand((B, N, Hkv, d), 5), _rand((B, N, Hkv, d), 6)
    G = Hq // Hkv
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)
    tk = torch.from_numpy(k).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    tv = torch.from_numpy(v).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    for causal in (True, False):
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal).permute(0, 2, 1, 3).numpy()
        out, lse = O.prefill_attn(q, k, v, causal=causal)          # default scale 1/sqrt(d), as the library's
        np.testing.assert_allclose(out, ref, rtol=0, atol=2e-6)
        s = (tq @ tk.transpose(-1, -2)) / math.sqrt(d)
        if causal:
            s = s.masked_fill(~torch.ones(N, N, dtype=torch.bool).tril(), float("-inf"))
        np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).numpy(), rtol=0, atol=2e-6)


def test_closed_forms():
    B, N, Hq, Hkv, d = 1, 9, 2, 1, 4
    k, v = _rand((B, N, Hkv, d), 7), _rand((B, N, Hkv, d), 8)
    # zero queries: uniform attention -> running mean of v, lse = log(number of visible keys)
    out, lse = O.prefill_attn(np.zeros((B, N, Hq, d)), k, v, causal=True)
    run_mean = np.cumsum(v[0, :, 0, :], axis=0) / np.arange(1, N + 1)[:, None]
    for h in range(Hq):
        np.testing.assert_allclose(out[0, :, h, :], run_mean, atol=2e-6)
        np.testing.assert_allclose(lse[0, h], np.log(np.arange(1, N + 1)), atol=2e-6)
    # constant v: every output row is that constant, whatever the logits; row 0 sees only key 0
    q = _rand((B, N, Hq, d), 9)
    out, _ = O.prefill_attn(q, k, np.full((B, N, Hkv, d), 2.5), causal=True)
    np.testing.assert_allclose(out, 2.5, atol=1e-6)
    out, lse = O.prefill_attn(q, k, v, scale=0.3, causal=True)
    np.testing.assert_allclose(out[0, 0, 1], v[0, 0, 0], atol=1e-6)
    np.testing.assert_allclose(lse[0, 1, 0], 0.3 * q[0, 0, 1] @ k[0, 0, 0], atol=1e-6)
    # a head reads KV head h // G: swapping the KV heads swaps the outputs of the two query-head groups
    k2, v2 = _rand((1, N, 2, d), 10), _rand((1, N, 2, d), 11)
    q2 = _rand((1, N, 4, d), 12)
    o1, l1 = O.prefill_attn(q2, k2, v2)
    o2, l2 = O.prefill_attn(q2[:, :, [2, 3, 0, 1]], k2[:, :, ::-1], v2[:, :, ::-1])
    np.testing.assert_allclose(o1[:, :, [2, 3, 0, 1]], o2, atol=1e-6)
    np.testing.assert_allclose(l1[:, [2, 3, 0, 1]], l2, atol=1e-6)


def test_normalisers_feed_the_score_oracle():
    """The scores computed from this function's normalisers equal the scores computed from scratch."""
    B, N, Hq, Hkv, d, T = 2, 41, 4, 2, 8, 6
    q, k, v = _rand((B, N, Hq, d), 13), _rand((B, N, Hkv, d), 14), _rand((B, N, Hkv, d), 15)
    _, lse = O.prefill_attn(q, k, v, scale=0.5)
    kw = dict(q_pos0=N - T, img_begin=5, n_img=25, scale=0.5, causal=True)
    sh0, sm0 = O.score_tokens(q[:, N - T:], k, **kw)
    sh1, sm1 = O.score_tokens(q[:, N - T:], k, row_lse=lse[:, :, N - T:], **kw)
    np.testing.assert_allclose(sh1, sh0, rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(sm1, sm0, rtol=1e-5, atol=1e-7)


def test_output_rounding():
    q, k, v = _rand((1, 5, 2, 4), 16), _rand((1, 5, 1, 4), 17), _rand((1, 5, 1, 4), 18)
    o32, _ = O.prefill_attn(q, k, v, dtype="f32")
    o16, _ = O.prefill_attn(q, k, v, dtype="bf16")
    assert o32.dtype == np.float32
    np.testing.assert_array_equal(o16, O.round_bf16(o16))
    np.testing.assert_allclose(o16, o32, rtol=2 ** -8)
