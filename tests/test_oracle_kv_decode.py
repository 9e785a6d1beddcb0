"""Pins for KV-cache compression (Sec. 3.2.2, App. A.2) and decode attention
over the retained cache: brute force, library routines, closed forms and the
"nothing to evict is an identity" invariants."""
import math

import numpy as np
import torch
import torch.nn.functional as F

from oracle import lvlm_oracle as O


# ---------------------------------------------------------------- threshold rule
def test_threshold_hand_example():
    # descending: .5, .25, .125(slot2), .125(slot3); total 1.0
    score = np.array([0.25, 0.5, 0.125, 0.125], dtype=np.float32)
    kind = np.full(4, O.KIND_IMAGE, dtype=np.uint8)
    assert O.kv_select_threshold(score, kind, 4, 0.5).tolist() == [False, True, False, False]
    assert O.kv_select_threshold(score, kind, 4, 0.75).tolist() == [True, True, False, False]
    assert O.kv_select_threshold(score, kind, 4, 0.8).tolist() == [True, True, True, False]   # tie: lower slot
    assert O.kv_select_threshold(score, kind, 4, 0.875).tolist() == [True, True, True, False]
    assert O.kv_select_threshold(score, kind, 4, 0.9).tolist() == [True] * 4
    assert O.kv_select_threshold(score, kind, 4, 1.0).tolist() == [True] * 4
    assert O.kv_select_threshold(score, kind, 4, 1e-9).tolist() == [False, True, False, False]  # at least one
    # a target a hair above an attainable sum needs one more entry (the target rounds up, never down)
    assert O.kv_select_threshold(score, kind, 4, 0.5 + 2.0 ** -40).tolist() == [True, True, False, False]


def test_threshold_matches_library_cumsum_on_dyadic_scores():
    rng = np.random.default_rng(0)
    for trial in range(20):
        L = int(rng.integers(1, 60))
        score = (rng.integers(0, 1 << 12, L) / float(1 << 12)).astype(np.float32)   # exact in fp
        kind = rng.choice([0, 1, 1, 1, 2], L).astype(np.uint8)
        beta = float(rng.choice([0.5, 0.9, 0.995, 0.25]))
        keep = O.kv_select_threshold(score, kind, L, beta)
        img = np.nonzero(kind == 1)[0]
        assert keep[kind != 1].all()                                         # text / generated stay
        if img.size == 0 or score[img].sum() == 0:
            assert keep.all()
            continue
        t = torch.from_numpy(score[img].astype(np.float64))
        order = torch.sort(t, descending=True, stable=True).indices
        cum = torch.cumsum(t[order], 0)
        target = beta * float(t.sum())
        n_kept = int((cum < target).sum()) + 1                                # shortest prefix reaching it
        expect = np.zeros(img.size, bool)
        expect[order[:n_kept].numpy()] = True
        assert np.array_equal(keep[img], expect)
        # minimality: dropping the last kept entry falls below the target
        if n_kept > 1:
            assert float(cum[n_kept - 2]) < target <= float(cum[n_kept - 1]) + 1e-12


def test_threshold_monotone_in_beta_and_prefix_property():
    rng = np.random.default_rng(1)
    L = 200
    score = rng.random(L).astype(np.float32) ** 6
    kind = np.full(L, 1, dtype=np.uint8)
    prev = None
    for beta in (0.1, 0.5, 0.9, 0.99, 0.995, 0.9999):
        keep = O.kv_select_threshold(score, kind, L, beta)
        assert score[keep].min() >= score[~keep].max() if (~keep).any() else True
        if prev is not None:
            assert (keep | ~prev).all()                                       # kept sets are nested
        prev = keep
    # spiky scores keep fewer entries than uniform ones at the same beta (Sec. 3.2.2)
    uniform = np.full(L, 0.01, dtype=np.float32)
    assert O.kv_select_threshold(uniform, kind, L, 0.995).sum() > O.kv_select_threshold(score, kind, L, 0.995).sum()
    assert O.kv_select_threshold(uniform, kind, L, 0.995).sum() == math.ceil(0.995 * L)


def test_threshold_degenerate_inputs():
    kind = np.array([1, 1, 0], dtype=np.uint8)
    assert O.kv_select_threshold(np.zeros(3, np.float32), kind, 3, 0.5).all()          # zero total
    assert O.kv_select_threshold(np.array([np.nan, 1.0, 5.0], np.float32), kind, 3, 0.5).tolist() == [False, True, True]
    assert O.kv_select_threshold(np.zeros(0, np.float32), np.zeros(0, np.uint8), 0, 0.5).size == 0
    assert O.score_fixed_point(np.array([0.5, -1.0, np.nan, 1e9])).tolist() == [1 << 31, 0, 0, 1 << 48]


# ---------------------------------------------------------------- budget rule
def _budget_brute(score, kind, L, budget, n_recent):
    if L <= budget:
        return [True] * L
    prot = [kind[s] == 0 or s >= L - n_recent for s in range(L)]
    ev = sorted([s for s in range(L) if not prot[s]], key=lambda s: (-float(score[s]), s))
    room = max(0, budget - sum(prot))
    kept = set(ev[:room])
    return [prot[s] or s in kept for s in range(L)]


def test_budget_matches_brute_force_and_counts():
    rng = np.random.default_rng(2)
    for trial in range(40):
        L = int(rng.integers(1, 50))
        score = (rng.integers(0, 8, L) / 8.0).astype(np.float32)
        kind = rng.choice([0, 1, 2], L, p=[0.2, 0.5, 0.3]).astype(np.uint8)
        budget = int(rng.integers(1, 55))
        n_recent = int(rng.integers(0, 4))
        keep = O.kv_select_budget(score, kind, L, budget, n_recent)
        assert keep.tolist() == _budget_brute(score, kind, L, budget, n_recent)
        prot = (kind == 0) | (np.arange(L) >= L - n_recent)
        assert keep[prot].all()
        if L > budget:
            assert keep.sum() == max(budget, prot.sum())
        else:
            assert keep.all()


# ---------------------------------------------------------------- compaction orders
def _fill_brute(keep):
    """Sequential simulation: walk holes from the left, survivors from beyond n'."""
    L = len(keep)
    n_new = sum(keep)
    slots = list(range(L))
    tail = [s for s in range(n_new, L) if keep[s]]
    for s in range(n_new):
        if not keep[s]:
            slots[s] = tail.pop(0)
    return slots[:n_new]


def test_compaction_orders():
    rng = np.random.default_rng(3)
    for trial in range(50):
        L = int(rng.integers(0, 40))
        keep = rng.random(L) < 0.6
        st = O.compaction_sources(keep, O.ORDER_STABLE)
        assert st.tolist() == [s for s in range(L) if keep[s]]
        fl = O.compaction_sources(keep, O.ORDER_FILL)
        assert fl.tolist() == _fill_brute(list(keep))
        assert sorted(fl.tolist()) == st.tolist()                              # same survivors
        assert all(fl[s] == s for s in range(len(fl)) if keep[s])              # survivors below n' stay
    keep = np.ones(10, bool)
    keep[3] = False                                                            # one eviction: one move
    assert O.compaction_sources(keep, O.ORDER_FILL).tolist() == [0, 1, 2, 9, 4, 5, 6, 7, 8]


def _make_cache(rng, B, Hkv, Lmax, d, lens):
    k = rng.standard_normal((B, Hkv, Lmax, d)).astype(np.float32)
    v = rng.standard_normal((B, Hkv, Lmax, d)).astype(np.float32)
    score = rng.random((B, Hkv, Lmax)).astype(np.float32)
    kind = rng.choice([0, 1, 2], (B, Hkv, Lmax)).astype(np.uint8)
    pos = np.tile(np.arange(Lmax, dtype=np.int32), (B, Hkv, 1))
    return k, v, score, kind, pos, np.array(lens, dtype=np.int32).reshape(B, Hkv)


def test_kv_compress_moves_all_arrays_together_and_identity_cases():
    rng = np.random.default_rng(4)
    B, Hkv, Lmax, d = 2, 2, 24, 4
    k, v, score, kind, pos, length = _make_cache(rng, B, Hkv, Lmax, d, [24, 10, 0, 17])
    for order in (O.ORDER_STABLE, O.ORDER_FILL):
        k2, v2, s2, kd2, p2, l2, nev = O.kv_compress(k, v, score, kind, pos, length, mode="threshold",
                                                     beta=0.6, order=order)
        assert np.array_equal(l2 + nev, length)
        for b in range(B):
            for g in range(Hkv):
                n = l2[b, g]
                src = p2[b, g, :n]                    # orig_pos was the slot number: tells where rows came from
                assert np.array_equal(k2[b, g, :n], k[b, g, src]) and np.array_equal(v2[b, g, :n], v[b, g, src])
                assert np.array_equal(s2[b, g, :n], score[b, g, src]) and np.array_equal(kd2[b, g, :n], kind[b, g, src])
                keep = O.kv_select_threshold(score[b, g], kind[b, g], int(length[b, g]), 0.6)
                assert sorted(src.tolist()) == np.nonzero(keep)[0].tolist()
    # beta >= 1 and budget >= len leave every array untouched
    for kw in (dict(mode="threshold", beta=1.0), dict(mode="budget", budget=24, n_recent=1)):
        res = O.kv_compress(k, v, score, kind, pos, length, **kw)
        for a, b_ in zip(res[:6], (k, v, score, kind, pos, length)):
            assert np.array_equal(a, b_)
        assert (res[6] == 0).all()
    # per-head independence: changing one head's scores does not change another head's result
    score_b = score.copy()
    score_b[0, 0] = rng.random(Lmax)
    r1 = O.kv_compress(k, v, score, kind, pos, length, mode="budget", budget=6, n_recent=1)
    r2 = O.kv_compress(k, v, score_b, kind, pos, length, mode="budget", budget=6, n_recent=1)
    assert np.array_equal(r1[4][0, 1], r2[4][0, 1]) and np.array_equal(r1[5][1], r2[5][1])


# ---------------------------------------------------------------- decode attention
def _decode_brute(q, kc, vc, length, scale):
    B, Hq, d = q.shape
    Hkv = kc.shape[1]
    G = Hq // Hkv
    out = np.zeros((B, Hq, d))
    probs = {}
    for b in range(B):
        for h in range(Hq):
            g = h // G
            L = int(length[b, g])
            logit = [scale * sum(float(q[b, h, c]) * float(kc[b, g, j, c]) for c in range(d)) for j in range(L)]
            mx = max(logit)
            den = sum(math.exp(x - mx) for x in logit)
            p = [math.exp(x - mx) / den for x in logit]
            probs[(b, h)] = p
            for c in range(d):
                out[b, h, c] = sum(p[j] * float(vc[b, g, j, c]) for j in range(L))
    return out, probs


def test_decode_brute_force_with_append_and_score_update():
    rng = np.random.default_rng(5)
    B, Hq, Hkv, d, Lmax = 2, 4, 2, 4, 12
    k, v, score, kind, pos, length = _make_cache(rng, B, Hkv, Lmax, d, [5, 11, 1, 8])
    q = rng.standard_normal((B, Hq, d))
    kn, vn = rng.standard_normal((B, Hkv, d)).astype(np.float32), rng.standard_normal((B, Hkv, d)).astype(np.float32)
    out, k2, v2, s2, kd2, p2, l2 = O.decode_attn(q, kn, vn, k, v, score, kind, pos, length, scale=0.5,
                                                 score_decay=0.5, new_pos=77)
    assert np.array_equal(l2, length + 1)
    for b in range(B):
        for g in range(Hkv):
            L = length[b, g]
            assert np.array_equal(k2[b, g, L], kn[b, g]) and np.array_equal(v2[b, g, L], vn[b, g])
            assert kd2[b, g, L] == O.KIND_GENERATED and p2[b, g, L] == 77
            assert np.array_equal(k2[b, g, :L], k[b, g, :L])
    ref, probs = _decode_brute(q, k2, v2, l2, 0.5)
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-7)
    G = Hq // Hkv
    for b in range(B):
        for g in range(Hkv):
            L = l2[b, g]
            old = score[b, g, :L].astype(np.float64).copy()
            old[L - 1] = 0.0                                                   # appended entry starts at 0
            pm = np.mean([probs[(b, h)] for h in range(g * G, (g + 1) * G)], axis=0)
            np.testing.assert_allclose(s2[b, g, :L], 0.5 * old + pm, rtol=1e-6)
            assert abs((s2[b, g, :L] - 0.5 * old).sum() - 1.0) < 1e-5          # probabilities sum to 1


def test_decode_closed_forms():
    rng = np.random.default_rng(6)
    B, Hq, Hkv, d, Lmax = 1, 2, 1, 8, 6
    k, v, score, kind, pos, _ = _make_cache(rng, B, Hkv, Lmax, d, [0])
    q = rng.standard_normal((B, Hq, d))
    one = np.array([[1]], dtype=np.int32)
    out = O.decode_attn(q, None, None, k, v, score, kind, pos, one)[0]
    np.testing.assert_allclose(out[0, 0], v[0, 0, 0], rtol=1e-6)               # one entry: o = v
    np.testing.assert_allclose(out[0, 1], v[0, 0, 0], rtol=1e-6)
    k_same = np.tile(k[:, :, :1], (1, 1, Lmax, 1))
    out = O.decode_attn(q, None, None, k_same, v, score, kind, pos, np.array([[Lmax]], dtype=np.int32))[0]
    np.testing.assert_allclose(out[0, 0], v[0, 0].mean(axis=0), rtol=1e-5, atol=1e-6)   # equal keys: mean(v)
    # empty cache, no append: output stays zero and nothing breaks
    out = O.decode_attn(q, None, None, k, v, score, kind, pos, np.array([[0]], dtype=np.int32))[0]
    assert (out == 0).all()


def test_decode_library_sdpa_cross_check():
    rng = np.random.default_rng(7)
    B, Hq, Hkv, d, L = 2, 6, 2, 16, 33
    k, v, score, kind, pos, length = _make_cache(rng, B, Hkv, L, d, [L] * (B * Hkv))
    q = rng.standard_normal((B, Hq, d))
    out = O.decode_attn(q, None, None, k, v, score, kind, pos, length, update_score=False)[0]
    tq = torch.from_numpy(q)[:, :, None, :]
    tk = torch.from_numpy(k.astype(np.float64)).repeat_interleave(Hq // Hkv, dim=1)
    tv = torch.from_numpy(v.astype(np.float64)).repeat_interleave(Hq // Hkv, dim=1)
    ref = F.scaled_dot_product_attention(tq, tk, tv)[:, :, 0].numpy()
    np.testing.assert_allclose(out, ref, rtol=1e-5, atol=1e-6)


def test_decode_is_unchanged_when_nothing_is_evicted_and_permutation_invariant():
    rng = np.random.default_rng(8)
    B, Hq, Hkv, d, Lmax = 1, 4, 2, 8, 20
    k, v, score, kind, pos, length = _make_cache(rng, B, Hkv, Lmax, d, [20, 13])
    q = rng.standard_normal((B, Hq, d))
    base = O.decode_attn(q, None, None, k, v, score, kind, pos, length)[0]
    for kw in (dict(mode="threshold", beta=1.0), dict(mode="budget", budget=20, n_recent=0)):
        c = O.kv_compress(k, v, score, kind, pos, length, **kw)
        again = O.decode_attn(q, None, None, *c[:6])[0]
        assert np.array_equal(again, base)                                     # bit-for-bit
    # STABLE and FILL hold the same survivors in different slots: same output up to reassociation
    a = O.kv_compress(k, v, score, kind, pos, length, mode="budget", budget=9, n_recent=1, order=O.ORDER_STABLE)
    b = O.kv_compress(k, v, score, kind, pos, length, mode="budget", budget=9, n_recent=1, order=O.ORDER_FILL)
    oa = O.decode_attn(q, None, None, *a[:6])[0]
    ob = O.decode_attn(q, None, None, *b[:6])[0]
    np.testing.assert_allclose(oa, ob, rtol=1e-5, atol=1e-6)
    assert not np.allclose(oa, base)                                           # eviction does change it
