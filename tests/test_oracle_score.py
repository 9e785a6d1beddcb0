"""Pins for oracle.score_tokens (Sec. 3.2.1: importance = attention received).

Each check is independent of the oracle's own code: brute-force Python loops,
a library softmax, closed forms and invariants of a row-stochastic matrix.
"""
import math

import numpy as np
import torch

from oracle import lvlm_oracle as O


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _brute_force(q, k, q_pos0, img_begin, n_img, scale, causal):
    """Explicit N x N-free loops: one probability at a time."""
    B, T, Hq, d = q.shape
    N, Hkv = k.shape[1], k.shape[2]
    G = Hq // Hkv
    head = [[[0.0] * n_img for _ in range(Hkv)] for _ in range(B)]
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for i in range(T):
                last = q_pos0 + i if causal else N - 1
                logits = []
                for j in range(min(last, N - 1) + 1):
                    logits.append(scale * sum(float(q[b, i, h, c]) * float(k[b, j, g, c]) for c in range(d)))
                mx = max(logits)
                den = sum(math.exp(x - mx) for x in logits)
                for j, x in enumerate(logits):
                    if img_begin <= j < img_begin + n_img:
                        head[b][g][j - img_begin] += math.exp(x - mx) / den / G
    head = np.array(head)
    return head, head.mean(axis=1)


def test_brute_force_causal_gqa():
    B, T, Hq, Hkv, d, N = 2, 3, 4, 2, 4, 9
    q, k = _rand((B, T, Hq, d), 1), _rand((B, N, Hkv, d), 2)
    kw = dict(q_pos0=N - T, img_begin=2, n_img=4, scale=0.7, causal=True)
    sh, sm = O.score_tokens(q, k, **kw)
    bh, bm = _brute_force(q, k, N - T, 2, 4, 0.7, True)
    np.testing.assert_allclose(sh, bh, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(sm, bm, rtol=1e-6, atol=1e-7)


def test_brute_force_noncausal_default_scale():
    B, T, Hq, Hkv, d, N = 1, 2, 6, 2, 8, 7
    q, k = _rand((B, T, Hq, d), 3), _rand((B, N, Hkv, d), 4)
    sh, sm = O.score_tokens(q, k, q_pos0=0, img_begin=0, n_img=N, causal=False)
    bh, bm = _brute_force(q, k, 0, 0, N, 1.0 / math.sqrt(d), False)
    np.testing.assert_allclose(sh, bh, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(sm, bm, rtol=1e-6, atol=1e-7)


def test_library_softmax_cross_check():
    B, T, Hq, Hkv, d, N = 2, 5, 8, 4, 16, 40
    q, k = _rand((B, T, Hq, d), 5), _rand((B, N, Hkv, d), 6)
    q_pos0 = N - T
    sh, sm = O.score_tokens(q, k, q_pos0=q_pos0, img_begin=3, n_img=30)
    tq, tk = torch.from_numpy(q), torch.from_numpy(k)
    tk = tk.repeat_interleave(Hq // Hkv, dim=2)                 # expand KV heads
    s = torch.einsum("bthd,bnhd->bhtn", tq, tk) / math.sqrt(d)
    mask = torch.arange(N)[None, :] > (q_pos0 + torch.arange(T))[:, None]
    s = s.masked_fill(mask, float("-inf"))
    col = torch.softmax(s, dim=-1).sum(dim=2)[:, :, 3:33]        # [B,Hq,30]
    ref_head = col.reshape(B, Hkv, Hq // Hkv, 30).mean(dim=2).numpy()
    np.testing.assert_allclose(sh, ref_head, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(sm, col.mean(dim=1).numpy(), rtol=1e-6, atol=1e-7)


def test_rows_are_stochastic_total_mass_is_T():
    # every softmax row sums to 1, so the column sums over ALL keys sum to T
    B, T, Hq, Hkv, d, N = 2, 6, 4, 2, 8, 20
    q, k = _rand((B, T, Hq, d), 7), _rand((B, N, Hkv, d), 8)
    sh, sm = O.score_tokens(q, k, q_pos0=N - T, img_begin=0, n_img=N)
    np.testing.assert_allclose(sh.sum(axis=-1), T, rtol=1e-6)
    np.testing.assert_allclose(sm.sum(axis=-1), T, rtol=1e-6)
    assert (sh >= 0).all() and (sm >= 0).all()


def test_identical_keys_closed_form():
    # all keys equal -> every visible key gets 1/(number visible) from each row
    B, T, Hq, Hkv, d, N = 1, 4, 2, 1, 8, 10
    q = _rand((B, T, Hq, d), 9)
    k = np.tile(_rand((1, 1, Hkv, d), 10), (B, N, 1, 1))
    q_pos0 = 6
    sh, sm = O.score_tokens(q, k, q_pos0=q_pos0, img_begin=0, n_img=N)
    expect = np.zeros(N)
    for i in range(T):
        vis = q_pos0 + i + 1
        expect[:vis] += 1.0 / vis
    np.testing.assert_allclose(sh[0, 0], expect, rtol=1e-6)
    np.testing.assert_allclose(sm[0], expect, rtol=1e-6)


def test_causal_mask_boundaries():
    B, T, Hq, Hkv, d, N = 1, 3, 2, 2, 4, 8
    q, k = _rand((B, T, Hq, d), 11), _rand((B, N, Hkv, d), 12)
    q_pos0 = 4                      # rows at 4,5,6; key 7 is never visible
    sh, _ = O.score_tokens(q, k, q_pos0=q_pos0, img_begin=0, n_img=N)
    assert (sh[..., 7] == 0).all()
    # key 6 is visible to the last row only: its column sum is below 1
    assert (sh[..., 6] > 0).all() and (sh[..., 6] < 1).all()
    # without the mask key 7 receives attention
    sh2, _ = O.score_tokens(q, k, q_pos0=q_pos0, img_begin=0, n_img=N, causal=False)
    assert (sh2[..., 7] > 0).all()


def test_permuting_keys_permutes_scores():
    B, T, Hq, Hkv, d, N = 1, 4, 4, 2, 8, 12
    q, k = _rand((B, T, Hq, d), 13), _rand((B, N, Hkv, d), 14)
    perm = np.random.default_rng(15).permutation(N)
    a, am = O.score_tokens(q, k, q_pos0=0, img_begin=0, n_img=N, causal=False)
    b, bm = O.score_tokens(q, k[:, perm], q_pos0=0, img_begin=0, n_img=N, causal=False)
    np.testing.assert_allclose(b, a[..., perm], rtol=1e-6)
    np.testing.assert_allclose(bm, am[..., perm], rtol=1e-6)


def test_softmax_shift_invariance_and_zero_scale():
    B, T, Hq, Hkv, d, N = 1, 3, 2, 1, 4, 6
    q, k = _rand((B, T, Hq, d), 16), _rand((B, N, Hkv, d), 17)
    # scale 0: all logits equal -> uniform over the N keys, column sum T/N
    sh, _ = O.score_tokens(q, k, q_pos0=0, img_begin=0, n_img=N, scale=0.0, causal=False)
    np.testing.assert_allclose(sh, T / N, rtol=1e-6)
    # duplicating a key splits nothing: both copies get the same score
    k2 = np.concatenate([k, k[:, :1]], axis=1)
    sh2, _ = O.score_tokens(q, k2, q_pos0=0, img_begin=0, n_img=N + 1, causal=False)
    assert np.array_equal(sh2[..., 0], sh2[..., N])


def test_one_hot_limit_counts_rows():
    # orthogonal keys, each query a large multiple of one key: P -> one-hot
    d, N = 8, 8
    k = np.eye(N, d)[None, :, None, :]                            # [1,N,1,d]
    target = [2, 2, 5, 0, 2]
    q = 200.0 * np.eye(N, d)[target][None, :, None, :]            # [1,T,1,d]
    sh, sm = O.score_tokens(q, k, q_pos0=0, img_begin=0, n_img=N, scale=1.0, causal=False)
    expect = np.bincount(target, minlength=N).astype(float)
    np.testing.assert_allclose(sh[0, 0], expect, atol=1e-6)
    np.testing.assert_allclose(sm[0], expect, atol=1e-6)


def test_head_reductions():
    # G = 1: score_head is per query head; score_mean is the mean over heads
    B, T, H, d, N = 1, 3, 4, 8, 10
    q, k = _rand((B, T, H, d), 18), _rand((B, N, H, d), 19)
    sh, sm = O.score_tokens(q, k, q_pos0=N - T, img_begin=1, n_img=6)
    np.testing.assert_allclose(sm, sh.mean(axis=1), rtol=1e-6)
    # a GQA group's score is the mean of what its query heads give alone
    Hq, Hkv = 4, 2
    k2 = _rand((B, N, Hkv, d), 20)
    sh2, _ = O.score_tokens(q, k2, q_pos0=N - T, img_begin=1, n_img=6)
    for g in range(Hkv):
        solo = [O.score_tokens(q[:, :, h:h + 1], k2[:, :, g:g + 1], q_pos0=N - T, img_begin=1,
                               n_img=6)[0][:, 0] for h in (2 * g, 2 * g + 1)]
        np.testing.assert_allclose(sh2[:, g], 0.5 * (solo[0] + solo[1]), rtol=1e-6)


def test_row_lse_path_matches():
    B, T, Hq, Hkv, d, N = 2, 4, 4, 2, 8, 15
    q, k = _rand((B, T, Hq, d), 21), _rand((B, N, Hkv, d), 22)
    q_pos0 = N - T
    tq, tk = torch.from_numpy(q), torch.from_numpy(k).repeat_interleave(2, dim=2)
    s = torch.einsum("bthd,bnhd->bhtn", tq, tk) / math.sqrt(d)
    mask = torch.arange(N)[None, :] > (q_pos0 + torch.arange(T))[:, None]
    lse = torch.logsumexp(s.masked_fill(mask, float("-inf")), dim=-1).numpy()   # [B,Hq,T]
    a = O.score_tokens(q, k, q_pos0=q_pos0, img_begin=2, n_img=8)
    b = O.score_tokens(q, k, q_pos0=q_pos0, img_begin=2, n_img=8, row_lse=lse)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-6)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-6)


def test_score_from_probs_agrees_with_the_pinned_path_and_closed_forms():
    # (1) probabilities built here with a library softmax give the scores of score_tokens (pinned above)
    rng = np.random.default_rng(41)
    B, T, Hq, Hkv, d, N, img0, n_img, q_pos0 = 2, 5, 6, 2, 8, 23, 3, 13, 18
    q, k = rng.standard_normal((B, T, Hq, d)), rng.standard_normal((B, N, Hkv, d))
    G = Hq // Hkv
    s = np.einsum("bthd,bnhd->bhtn", q, np.repeat(k, G, axis=2)) / math.sqrt(d)
    mask = np.arange(N)[None, :] > (q_pos0 + np.arange(T))[:, None]
    p = torch.softmax(torch.from_numpy(np.where(mask, -np.inf, s)), dim=-1).numpy()
    sh, sm = O.score_from_probs(p, n_kv_heads=Hkv, img_begin=img0, n_img=n_img)
    rh, rm = O.score_tokens(q, k, q_pos0=q_pos0, img_begin=img0, n_img=n_img)
    assert np.allclose(sh, rh, rtol=1e-6, atol=1e-7) and np.allclose(sm, rm, rtol=1e-6, atol=1e-7)
    # (2) one probability at a time
    for b, g, j in ((0, 0, 0), (1, 1, 12), (0, 1, 5)):
        want = sum(p[b, g * G + h, i, img0 + j] for h in range(G) for i in range(T)) / G
        assert abs(sh[b, g, j] - want) < 1e-6
    # (3) uniform rows: every key receives T / N from every head; one-hot rows: the hit column counts the rows
    u = np.full((1, 4, 7, 10), 0.1)
    sh, sm = O.score_from_probs(u, n_kv_heads=2, img_begin=2, n_img=6)
    assert np.allclose(sh, 0.7) and np.allclose(sm, 0.7)
    e = np.zeros((1, 4, 7, 10))
    e[..., 4] = 1.0
    sh, sm = O.score_from_probs(e, n_kv_heads=4, img_begin=2, n_img=6)
    assert np.allclose(sh[0, :, 2], 7.0) and np.allclose(np.delete(sh, 2, axis=2), 0.0) and sm[0, 2] == 7.0
