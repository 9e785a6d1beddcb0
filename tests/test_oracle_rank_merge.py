"""Pins for the ordering, partition, merge rule, compaction and schedule
(Sec. 3.2.1 par. 4; App. A.2).  Brute force with exact rationals, library
sorts, closed forms and counting invariants."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import lvlm_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- rounding
def _bf16_exact(x: float) -> float:
    """Nearest bf16 (8 significant bits) by exact rational arithmetic, ties to even."""
    if x == 0:
        return 0.0
    fx = Fraction(x)
    sign = -1 if fx < 0 else 1
    fx = abs(fx)
    e = 0
    while fx >= 2:
        fx /= 2
        e += 1
    while fx < 1:
        fx *= 2
        e -= 1
    scaled = fx * 128                      # 1.xxxxxxx with 7 fraction bits
    lo = scaled.numerator // scaled.denominator
    rem = scaled - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return float(sign * Fraction(lo, 128) * Fraction(2) ** e)


def test_round_bf16_matches_exact_rounding_and_torch():
    rng = np.random.default_rng(0)
    xs = list(rng.standard_normal(200) * 10.0 ** rng.integers(-3, 4, 200))
    # a value just above a tie that a float64 -> float32 -> bf16 chain gets wrong
    xs += [1.0 + 2.0 ** -8 + 2.0 ** -30, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8 + 2.0 ** -40)]
    got = O.round_bf16(np.array(xs))
    for x, g in zip(xs, got):
        assert float(g) == _bf16_exact(float(x)), x
    f32 = rng.standard_normal(1000).astype(np.float32)
    ref = torch.from_numpy(f32).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.round_bf16(f32.astype(np.float64)), ref)


# ---------------------------------------------------------------- ordering
def test_rank_matches_python_sort_and_torch_stable_sort():
    rng = np.random.default_rng(1)
    for n in (1, 2, 17, 300):
        s = rng.integers(0, 6, n).astype(np.float32) / 4.0       # many ties
        order = O.order_desc(s)
        assert list(order) == sorted(range(n), key=lambda j: (-float(s[j]), j))
        t = torch.sort(torch.from_numpy(s), descending=True, stable=True).indices.numpy()
        assert np.array_equal(order, t)
        rank = O.rank_desc(s)
        assert sorted(rank) == list(range(n))
        assert all(order[rank[j]] == j for j in range(n))


def test_rank_special_values():
    s = np.array([0.0, np.nan, -0.0, np.inf, -np.inf, 1.0, np.nan, 1.0], dtype=np.float32)
    # inf, then the two 1.0 (index order), then the zeros (equal, index order), -inf, NaNs last
    assert list(O.order_desc(s)) == [3, 5, 7, 0, 2, 4, 1, 6]


def test_partition_counts_and_sets():
    rng = np.random.default_rng(2)
    n = 50
    s = rng.random(n).astype(np.float32)
    for n_keep in (1, 2, 25, 49):
        keep, merged = O.partition(s, n_keep)
        r = n - n_keep
        assert len(keep) == n - (r + 1) and len(merged) == r + 1        # Sec. 3.2.1 sizes
        assert sorted(set(keep) | set(merged)) == list(range(n))
        assert list(keep) == sorted(keep)
        assert min(s[keep], default=np.inf) >= max(s[merged])
        assert all(s[merged[i]] >= s[merged[i + 1]] for i in range(r))   # least important last
    keep, merged = O.partition(s, n)                                      # r = 0: nothing merged
    assert list(keep) == list(range(n)) and len(merged) == 0


def test_partition_tie_break_prefers_lower_index():
    s = np.array([0.5, 0.5, 0.5, 0.5], dtype=np.float32)
    keep, merged = O.partition(s, 3)
    assert list(keep) == [0, 1] and list(merged) == [2, 3]


# ---------------------------------------------------------------- merge rule
def _pairwise_fraction_weights(m):
    """Run the paper's loop symbolically on unit vectors with exact rationals."""
    queue = [[Fraction(int(i == j)) for j in range(m)] for i in range(m)]
    while len(queue) > 1:
        last, prev = queue.pop(), queue.pop()
        queue.append([(a + b) / 2 for a, b in zip(prev, last)])
    return queue[0]


@pytest.mark.parametrize("m", [1, 2, 3, 7, 20])
def test_pairwise_weights_equal_the_iterated_loop(m):
    w = O.merge_weights(O.MERGE_PAIRWISE, m)
    assert [Fraction(float(x)) for x in w] == _pairwise_fraction_weights(m)
    rows = np.random.default_rng(m).integers(-8, 8, (m, 5)).astype(np.float64)
    assert np.array_equal(O.merge_pairwise_loop(rows), w @ rows)       # dyadic: exact


def test_linear_rank_weights():
    assert np.allclose(O.merge_weights(O.MERGE_LINEAR_RANK, 2), [2 / 3, 1 / 3])
    assert np.allclose(O.merge_weights(O.MERGE_LINEAR_RANK, 1), [1.0])
    for m in (3, 10, 1413, 11294):
        w = O.merge_weights(O.MERGE_LINEAR_RANK, m)
        raw = O.merge_weights(O.MERGE_LINEAR_RAW, m)
        assert list(raw[:2]) == [m, m - 1] and raw[-1] == 1            # W_v = {r+1, r, ..., 1}
        assert abs(w.sum() - 1.0) < 1e-12
        np.testing.assert_allclose(w * raw.sum(), raw, rtol=1e-12)
        assert (np.diff(w) < 0).all()                                  # most important weighs most


def test_merge_compact_hand_worked_example():
    # 1 system row, 5 image rows, 1 text row; keep 3 of the 5 image tokens (r = 2)
    score = np.array([[0.10, 0.40, 0.05, 0.30, 0.15]], dtype=np.float32)
    hid = np.array([[[9, 9], [1, 10], [2, 20], [3, 30], [4, 40], [5, 50], [7, 7]]], dtype=np.float64)
    pos = np.arange(7, dtype=np.int32).reshape(1, 7, 1)
    outs, keep, merged = O.merge_compact([hid, pos], score, img_begin=1, n_img=5, n_keep=3,
                                         rules=[O.RULE_WEIGHTED, O.RULE_TOP], dtypes=["f32", "f32"])
    # descending: tok1 (.40), tok3 (.30), tok4 (.15), tok0 (.10), tok2 (.05)
    assert keep.tolist() == [[1, 3]] and merged.tolist() == [[4, 0, 2]]
    w = [Fraction(3, 6), Fraction(2, 6), Fraction(1, 6)]
    new = [float(w[0] * 5 + w[1] * 1 + w[2] * 3), float(w[0] * 50 + w[1] * 10 + w[2] * 30)]
    expect = np.array([[[9, 9], [2, 20], [4, 40], new, [7, 7]]])
    np.testing.assert_allclose(outs[0], expect, rtol=1e-7)
    assert outs[1][0, :, 0].tolist() == [0, 2, 4, 5, 6]       # position of the rank-0 merged token
    # explicit table: the iterated pairwise rule gives 1/2, 1/4, 1/4
    outs2, _, _ = O.merge_compact([hid], score, img_begin=1, n_img=5, n_keep=3,
                                  w=O.merge_weights(O.MERGE_PAIRWISE, 3))
    np.testing.assert_allclose(outs2[0][0, 3], [0.5 * 5 + 0.25 * 1 + 0.25 * 3, 0.5 * 50 + 0.25 * 10 + 0.25 * 30])


def test_merge_compact_invariants():
    rng = np.random.default_rng(3)
    B, n_sys, n_img, n_txt, C = 2, 3, 40, 4, 6
    N = n_sys + n_img + n_txt
    hid = rng.standard_normal((B, N, C))
    score = rng.random((B, n_img)).astype(np.float32)
    for n_keep in (1, 7, 39):
        r = n_img - n_keep
        (out,), keep, merged = O.merge_compact([hid], score, img_begin=n_sys, n_img=n_img, n_keep=n_keep)
        assert out.shape == (B, N - r, C)                                # length N - r
        assert np.array_equal(out[:, :n_sys], hid[:, :n_sys])            # text never touched
        assert np.array_equal(out[:, n_sys + n_keep:], hid[:, n_sys + n_img:])
        for b in range(B):
            img = hid[b, n_sys:n_sys + n_img]
            assert np.array_equal(out[b, n_sys:n_sys + n_keep - 1], img[keep[b]])
            pm = img[merged[b]]
            new = out[b, n_sys + n_keep - 1]
            assert (new <= pm.max(axis=0) + 1e-6).all() and (new >= pm.min(axis=0) - 1e-6).all()
    # r = 0: bit-for-bit identity
    (out,), keep, merged = O.merge_compact([hid], score, img_begin=n_sys, n_img=n_img, n_keep=n_img)
    assert np.array_equal(out, hid) and merged.shape == (B, 0)
    # constant image rows map to themselves
    const = hid.copy()
    const[:, n_sys:n_sys + n_img] = 1.25
    (out,), _, _ = O.merge_compact([const], score, img_begin=n_sys, n_img=n_img, n_keep=5)
    np.testing.assert_allclose(out[:, n_sys:n_sys + 5], 1.25, rtol=1e-6)


def test_merge_compact_bf16_output_is_representable():
    rng = np.random.default_rng(4)
    hid = torch.from_numpy(rng.standard_normal((1, 20, 8)).astype(np.float32)).to(torch.bfloat16)
    hid = hid.to(torch.float32).numpy()
    score = rng.random((1, 20)).astype(np.float32)
    (out,), _, _ = O.merge_compact([hid], score, img_begin=0, n_img=20, n_keep=4, dtypes=["bf16"])
    rt = torch.from_numpy(out).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(rt, out)


# ---------------------------------------------------------------- similarity merge (ours)
def test_similarity_merge_conserves_mass_and_assigns_nearest():
    rng = np.random.default_rng(5)
    n, C, n_keep = 30, 6, 7
    centres = rng.standard_normal((n_keep, C)) * 3
    which = rng.integers(0, n_keep, n)
    which[:n_keep] = np.arange(n_keep)
    hid = centres[which] + 0.01 * rng.standard_normal((n, C))
    size = rng.integers(1, 4, n).astype(np.float64)
    score = np.zeros(n, dtype=np.float32)
    score[:n_keep] = 1.0                                   # the first copy of each centre dominates
    rows, new_size, dom, assign = O.merge_similarity(hid, size, score, n_keep)
    assert list(dom) == list(range(n_keep))
    assert list(assign) == list(which[n_keep:])            # clustered data: nearest = own centre
    np.testing.assert_allclose((rows * new_size[:, None]).sum(0), (hid * size[:, None]).sum(0), rtol=1e-5)
    assert abs(new_size.sum() - size.sum()) < 1e-6
    # brute-force cosine argmax
    for t, a in zip(range(n_keep, n), assign):
        cos = [float(hid[t] @ hid[i] / np.linalg.norm(hid[t]) / np.linalg.norm(hid[i])) for i in dom]
        assert int(np.argmax(cos)) == a


def test_merge_similar_batch_planes_and_identity():
    rng = np.random.default_rng(6)
    B, n_sys, n_img, n_txt, C, n_keep = 2, 2, 24, 3, 5, 6
    N = n_sys + n_img + n_txt
    hid = rng.standard_normal((B, N, C))
    ids = np.arange(B * N, dtype=np.int32).reshape(B, N, 1)
    score = rng.random((B, n_img)).astype(np.float32)
    size = rng.integers(1, 4, (B, n_img)).astype(np.float64)
    (out, oid), keep, assign, new_size = O.merge_similar([hid, ids], score, img_begin=n_sys, n_img=n_img,
                                                         n_keep=n_keep, size=size, rules=[O.RULE_WEIGHTED, O.RULE_TOP])
    assert out.shape == (B, N - (n_img - n_keep), C)
    assert np.array_equal(out[:, :n_sys], hid[:, :n_sys]) and np.array_equal(out[:, n_sys + n_keep:], hid[:, n_sys + n_img:])
    for b in range(B):
        img = hid[b, n_sys:n_sys + n_img]
        rows, ns, dom, a_rest = O.merge_similarity(img, size[b], score[b], n_keep)       # the one-row form agrees
        np.testing.assert_allclose(out[b, n_sys:n_sys + n_keep], rows, rtol=1e-6)
        assert np.array_equal(keep[b], dom) and np.allclose(new_size[b], ns)
        assert list(keep[b]) == sorted(np.argsort(-score[b], kind="stable")[:n_keep])     # dominant = top scores
        assert all(assign[b, keep[b][p]] == p for p in range(n_keep))
        # size-weighted mass is conserved per channel, and sizes add up
        np.testing.assert_allclose((out[b, n_sys:n_sys + n_keep] * new_size[b][:, None]).sum(0),
                                   (img * size[b][:, None]).sum(0), rtol=1e-5, atol=1e-6)
        assert abs(new_size[b].sum() - size[b].sum()) < 1e-6
        assert np.array_equal(oid[b, n_sys:n_sys + n_keep, 0], ids[b, n_sys + keep[b], 0])  # ids of the dominant tokens
    # an imposed assignment is honoured
    forced = np.zeros((B, n_img), dtype=np.int32)
    (out2, _), _, a2, ns2 = O.merge_similar([hid, ids], score, img_begin=n_sys, n_img=n_img, n_keep=n_keep,
                                            assign=forced, rules=[O.RULE_WEIGHTED, O.RULE_TOP])
    np.testing.assert_allclose(out2[:, n_sys], hid[:, n_sys:n_sys + n_img].mean(axis=1), rtol=1e-6)
    assert (ns2[:, 0] == n_img).all() and (ns2[:, 1:] == 0).all()
    # n_keep == n_img: nothing changes
    (out3, _), keep3, _, ns3 = O.merge_similar([hid, ids], score, img_begin=n_sys, n_img=n_img, n_keep=n_img)
    assert np.array_equal(out3, hid) and (ns3 == 1).all() and list(keep3[0]) == list(range(n_img))


# ---------------------------------------------------------------- schedule
def test_schedule_golden_and_properties():
    with open(os.path.join(GOLDEN, "paper_constants.json")) as f:
        gold = json.load(f)
    for n_img, f in [(2048, 0.03), (2048, 0.35), (2048, 0.15), (1792, 0.35), (16384, 0.03), (1476, 0.03)]:
        s = O.schedule(n_img, f, 3)
        assert s[-1] == int(n_img * f + 0.5)                   # the budget is met at the last stage
        assert s[0] >= s[1] >= s[2] >= 1
        ratio = f ** (1 / 3)                                    # constant reduction ratio (App. A.2)
        for prev, cur in zip([n_img] + s[:-1], s):
            assert abs(cur / prev - ratio) < 2.0 / prev + 1e-3
    assert O.schedule(2048, 1.0, 3) == [2048, 2048, 2048]
    assert O.schedule(576, 0.5, 1) == [288]
    assert O.schedule(10, 1e-9, 3) == [1, 1, 1]
    assert gold["merge_layers_qwen25vl_7b"] == [5, 9, 13] and gold["kv_beta"] == 0.995
    assert gold["keep_budgets"] == [0.35, 0.15, 0.03]


def _stage_count_exact(n, f_num, f_den, s, S=3):
    """floor(n * (f_num/f_den)^(s/S) + 1/2) without floating point: k is that value exactly when
    (2k-1)^S * f_den^s <= (2n)^S * f_num^s < (2k+1)^S * f_den^s."""
    rhs = (2 * n) ** S * f_num ** s
    k = 0
    while (2 * k + 1) ** S * f_den ** s <= rhs:
        k += 1
    return k


def test_schedule_every_stage_is_rounded_half_up_from_the_original_count():
    """App. A.2: a constant reduction ratio per merge layer, fixed by the budget.  The counts of every stage (not
    only the last) are round-half-up of n * f^(s/3) taken from the ORIGINAL count: the printed table below was
    evaluated by hand for the benchmark shapes, and the integer-cube bracket gives the same values with no
    floating point at all, so a floor instead of a round, or a ratio applied to the previous stage's rounded
    count, fails here (1792 * 0.35^(2/3) = 889.97 must give 890; 636 * 0.3107 = 197.6 -> 198 only from 2048)."""
    table = {(2048, 3, 100): [636, 198, 61], (2048, 35, 100): [1443, 1017, 717], (1792, 35, 100): [1263, 890, 627],
             (16384, 3, 100): [5091, 1582, 492]}
    for (n, a, b), want in table.items():
        assert O.schedule(n, a / b, 3) == want
        assert [_stage_count_exact(n, a, b, s) for s in (1, 2, 3)] == want
    for n, a, b in [(2048, 15, 100), (1476, 3, 100), (4096, 1, 8), (999, 1, 2), (7, 1, 3)]:
        assert O.schedule(n, a / b, 3) == [max(1, _stage_count_exact(n, a, b, s)) for s in (1, 2, 3)]
    assert O.schedule(576, 0.5, 1) == [288]
