"""CPU oracle for the LightVLM token-reduction path (arXiv 2509.00419).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
path computes, written from the paper (Sec. 3.2.1 "Pyramid token merging",
Sec. 3.2.2 "KV Cache compression", App. A.2 "Model Settings").  It shares no
code with the HIP library and never imports it; only tests, the smoke check and
the bench's cpu_baseline leg may call it.

Conventions
-----------
* Every floating-point input arrives as a numpy array that already holds the
  values the GPU sees (bf16 / fp32 inputs widened exactly to float64).
* All arithmetic is float64; an output is rounded once, at the very end, to the
  dtype the GPU writes ("f32" or "bf16", round-to-nearest-even).
* Integer work (ranks, index lists, cumulative thresholds, slot moves) is exact.
* No blocking, fusion or reordering beyond what each definition states.

Pins (tests/test_oracle_*.py): every function below is checked against
brute-force pure-Python loops on tiny inputs, closed forms, invariants and
library routines (torch.softmax / torch.sort / torch.cumsum /
scaled_dot_product_attention in fp64).  The similarity merge (merge_similarity)
and the fixed-budget eviction (kv_select_budget) are not defined by the paper
at all: their definitions are this build's and are pinned only by brute force
and invariants ("parity unpinned" by the paper).
"""
from __future__ import annotations

import math

import numpy as np

# --------------------------------------------------------------------------
# rounding helpers
# --------------------------------------------------------------------------


def round_bf16(x) -> np.ndarray:
    """float64 -> nearest bfloat16 (ties to even), returned as float32 values.

    Two-step: float64 -> float32 with round-to-odd (truncate toward zero and
    set the last bit when inexact), then float32 -> bf16 with ties-to-even.
    Round-to-odd in the first step makes the double rounding exact.
    """
    x = np.asarray(x, dtype=np.float64)
    f = x.astype(np.float32)                       # nearest-even first guess
    back = f.astype(np.float64)
    inexact = np.isfinite(x) & (back != x)
    # move the guess toward zero when it overshot in magnitude
    over = inexact & (np.abs(back) > np.abs(x))
    f = np.where(over, np.nextafter(f, np.float32(0.0)), f).astype(np.float32)
    bits = f.view(np.uint32).copy()
    bits = np.where(inexact, bits | np.uint32(1), bits).astype(np.uint32)
    # float32 -> bf16, ties to even, on the bit pattern
    nan = np.isnan(x)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    rounded = np.where(nan, np.uint32(0x7FC00000), rounded).astype(np.uint32)
    return rounded.view(np.float32).reshape(x.shape)


def round_out(x, dtype: str) -> np.ndarray:
    """Round a float64 result to the output dtype; returns float32 values."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "bf16":
        return round_bf16(x)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# step 1: token importance = attention received   (Sec. 3.2.1, par. 2-3)
# --------------------------------------------------------------------------


def score_tokens(q, k, *, q_pos0: int, img_begin: int, n_img: int,
                 scale: float | None = None, causal: bool = True,
                 row_lse=None):
    """Attention each image key receives from the query rows.

    q: [B, T, Hq, d]   query rows; row i sits at absolute position q_pos0 + i
    k: [B, N, Hkv, d]  keys of the whole sequence
    For head h (KV head g = h // G, G = Hq // Hkv) and row i the softmax runs
    over every key j the row may see (j <= q_pos0 + i when causal, else all N),
    system, image and text keys alike.  The importance of key j under head h
    is the column sum over the T rows of those probabilities -- the "cumsum
    attention score" A in R^N of Sec. 3.2.1.  score_head averages the G query
    heads of a KV group (Sec. 3.2.2 prunes per head); score_mean averages the
    KV groups, i.e. all heads (Sec. 3.2.1: "averaged ... across heads").

    row_lse (optional) [B, Hq, T]: natural-log sum-exp of each row's scaled
    logits, as an attention kernel would hand over; used instead of
    recomputing the row normaliser.

    Returns (score_head [B,Hkv,n_img] f32, score_mean [B,n_img] f32).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    B, T, Hq, d = q.shape
    Bk, N, Hkv, dk = k.shape
    assert B == Bk and d == dk and Hq % Hkv == 0
    assert 0 <= img_begin and img_begin + n_img <= N
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    scale = float(scale)
    score_head = np.zeros((B, Hkv, n_img), dtype=np.float64)
    pos = q_pos0 + np.arange(T)
    visible = (np.arange(N)[None, :] <= pos[:, None]) if causal else np.ones((T, N), bool)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            s = scale * (q[b, :, h, :] @ k[b, :, g, :].T)          # [T, N]
            s = np.where(visible, s, -np.inf)
            if row_lse is None:
                m = s.max(axis=1, keepdims=True)
                e = np.exp(s - m)
                p = e / e.sum(axis=1, keepdims=True)
            else:
                lse = np.asarray(row_lse, dtype=np.float64)[b, h, :, None]
                p = np.exp(s - lse)
            a = p.sum(axis=0)                                      # column sums, [N]
            score_head[b, g] += a[img_begin:img_begin + n_img]
        score_head[b] /= G
    score_mean = score_head.sum(axis=1) / Hkv
    return score_head.astype(np.float32), score_mean.astype(np.float32)


def score_from_probs(probs, *, n_kv_heads: int, img_begin: int, n_img: int):
    """The same scores when the attention probabilities are already there (Sec. 3.2.2 takes them from "the
    full attention matrix" of a plain attention just as well): probs [B, Hq, T, N], the softmax rows of the T
    query rows to be summed.  Column sums over the rows, mean over the G heads of a KV group, mean over the
    groups.  Returns (score_head [B,Hkv,n_img] f32, score_mean [B,n_img] f32)."""
    p = np.asarray(probs, dtype=np.float64)
    B, Hq, T, N = p.shape
    assert Hq % n_kv_heads == 0 and 0 <= img_begin and img_begin + n_img <= N
    G = Hq // n_kv_heads
    a = p[:, :, :, img_begin:img_begin + n_img].sum(axis=2)            # [B, Hq, n_img]: attention received
    score_head = a.reshape(B, n_kv_heads, G, n_img).sum(axis=2) / G
    score_mean = score_head.sum(axis=1) / n_kv_heads
    return score_head.astype(np.float32), score_mean.astype(np.float32)


def prefill_attn(q, k, v, *, scale: float | None = None, causal: bool = True, dtype: str = "f32"):
    """Prefill self-attention of one layer, with the row normalisers it leaves behind.

    q: [B, N, Hq, d], k, v: [B, N, Hkv, d] (row i of q sits at position i).  Head h reads KV head h // G.
    out[b,i,h,:] = sum_j softmax_j(scale * q[b,i,h].k[b,j,g]) v[b,j,g,:] over the keys row i may see (j <= i
    when causal, else all N) -- the attention the paper's scores are a by-product of (Sec. 3.2.1: the
    scores come "from the attention" of the layer, Sec. 3.2.2: from its kernel's statistics).
    lse[b,h,i] is the natural-log sum-exp of row i's scaled logits over those keys: with it,
    score_tokens(..., row_lse=lse[:, :, N-T:]) gives the scores of the last T rows without a second
    normaliser pass.

    Returns (out [B,N,Hq,d] rounded to `dtype`, lse [B,Hq,N] f32).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, N, Hq, d = q.shape
    Hkv = k.shape[2]
    assert k.shape == (B, N, Hkv, d) and v.shape == (B, N, Hkv, d) and Hq % Hkv == 0
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    scale = float(scale)
    out = np.zeros((B, N, Hq, d), dtype=np.float64)
    lse = np.zeros((B, Hq, N), dtype=np.float64)
    visible = (np.arange(N)[None, :] <= np.arange(N)[:, None]) if causal else np.ones((N, N), bool)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            s = scale * (q[b, :, h, :] @ k[b, :, g, :].T)          # [N, N]
            s = np.where(visible, s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            den = e.sum(axis=1, keepdims=True)
            out[b, :, h, :] = (e / den) @ v[b, :, g, :]
            lse[b, h, :] = (m + np.log(den))[:, 0]
    return round_out(out, dtype), lse.astype(np.float32)


# --------------------------------------------------------------------------
# step 2: order by importance   (Sec. 3.2.1, par. 4: "reorder ... by importance")
# --------------------------------------------------------------------------


def rank_desc(s) -> np.ndarray:
    """rank[j] = number of entries that come before j in descending order.

    i precedes j when s_i > s_j, or s_i == s_j and i < j (lower index first).
    NaN is placed below every number (NaNs tie with each other).  Written as
    the counting definition, O(n^2), in row chunks to bound memory.
    """
    s = np.asarray(s, dtype=np.float64).ravel()
    n = s.shape[0]
    nan = np.isnan(s)
    v = np.where(nan, -np.inf, s)
    # tier: 1 for numbers, 0 for NaN, so that -inf still beats NaN
    tier = (~nan).astype(np.int8)
    idx = np.arange(n)
    rank = np.zeros(n, dtype=np.int64)
    step = max(1, (1 << 22) // max(n, 1))
    for j0 in range(0, n, step):
        j1 = min(n, j0 + step)
        vj, tj, ij = v[j0:j1, None], tier[j0:j1, None], idx[j0:j1, None]
        greater = (tier[None, :] > tj) | ((tier[None, :] == tj) & (v[None, :] > vj))
        equal = (tier[None, :] == tj) & (v[None, :] == vj)
        rank[j0:j1] = (greater | (equal & (idx[None, :] < ij))).sum(axis=1)
    return rank


def order_desc(s) -> np.ndarray:
    """Indices listed from most to least important (inverse of rank_desc)."""
    rank = rank_desc(s)
    order = np.empty_like(rank)
    order[rank] = np.arange(rank.shape[0])
    return order


def partition(score, n_keep: int):
    """Split one row of image-token scores into P_unmerged and P_merged.

    Sec. 3.2.1: with r tokens to remove, P_unmerged holds the N-(r+1)
    highest-scoring tokens and P_merged the other r+1, ordered by importance
    (least important last).  n_keep = N - r counts the merged slot.
    Returns (keep_idx ascending [n_keep-1], merged_idx in rank order [r+1]).
    r == 0 means no reduction was asked for: keep everything, merge nothing.
    """
    score = np.asarray(score)
    n = score.shape[0]
    assert 1 <= n_keep <= n
    if n_keep == n:
        return np.arange(n, dtype=np.int32), np.zeros(0, dtype=np.int32)
    order = order_desc(score)
    keep = np.sort(order[:n_keep - 1]).astype(np.int32)
    merged = order[n_keep - 1:].astype(np.int32)
    return keep, merged


# --------------------------------------------------------------------------
# step 3a: the paper's merge rule   (Sec. 3.2.1, par. 4)
# --------------------------------------------------------------------------

MERGE_LINEAR_RANK = 0   # W_v = {r+1, ..., 1} normalised to sum 1 (default)
MERGE_PAIRWISE = 1      # closed form of the iterated equal-weight tail merge
MERGE_LINEAR_RAW = 2    # W_v exactly as printed, not normalised


def merge_weights(mode: int, m: int) -> np.ndarray:
    """Rank -> weight table for the m = r+1 merged tokens (rank 0 = most important).

    LINEAR_RANK: w_k = (m-k) / (m(m+1)/2)  -- the printed weight list W_v,
      scaled so the merged token keeps the scale of a hidden state.
    PAIRWISE: the loop "replace the last two queue entries by their
      equal-weight mean" run until one entry is left gives w_k = 2^-(k+1) for
      k < m-1 and w_{m-1} = 2^-(m-1).
    LINEAR_RAW: w_k = m - k.
    """
    k = np.arange(m, dtype=np.float64)
    if mode == MERGE_LINEAR_RANK:
        return (m - k) / (m * (m + 1) / 2.0)
    if mode == MERGE_PAIRWISE:
        w = np.ldexp(1.0, -(np.arange(m) + 1)).astype(np.float64)
        if m >= 1:
            w[m - 1] = math.ldexp(1.0, -(m - 1))
        return w
    if mode == MERGE_LINEAR_RAW:
        return m - k
    raise ValueError("unknown merge mode")


def merge_pairwise_loop(rows) -> np.ndarray:
    """The iterative definition: combine the last two queue entries with equal
    weights until one remains.  rows: [m, C] in rank order."""
    queue = [np.asarray(r, dtype=np.float64) for r in rows]
    while len(queue) > 1:
        last = queue.pop()
        prev = queue.pop()
        queue.append(0.5 * prev + 0.5 * last)
    return queue[0]


RULE_WEIGHTED = 0   # P_new = sum_k w_k * P_merged[k]
RULE_TOP = 1        # P_new = entry of the rank-0 merged token (ids, positions)


def merge_compact(planes, score_mean, *, img_begin: int, n_img: int, n_keep: int,
                  w=None, rules=None, dtypes=None):
    """Steps 2-4 for a batch: partition, merge, and compact every plane.

    planes: list of arrays [B, N, row_elems] that share the token axis
            (hidden states, optionally this layer's K and V, position ids).
    score_mean: [B, n_img].
    w: optional rank->weight table of length r+1 (values used as given);
       default LINEAR_RANK.
    Output row order (Sec. 3.2.1: P_compressed = [P_unmerged, P_new]): rows
    before the image span, P_unmerged in ascending original index, P_new,
    rows after the image span.
    Returns (out_planes, keep_idx [B, n_keep-1], merged_idx [B, r+1]).
    """
    score_mean = np.asarray(score_mean)
    B = score_mean.shape[0]
    r = n_img - n_keep
    rules = rules or [RULE_WEIGHTED] * len(planes)
    dtypes = dtypes or ["f32"] * len(planes)
    if r == 0:
        outs = [np.array(p, copy=True) for p in planes]
        keep = np.tile(np.arange(n_img, dtype=np.int32), (B, 1))
        return outs, keep, np.zeros((B, 0), dtype=np.int32)
    m = r + 1
    wt = merge_weights(MERGE_LINEAR_RANK, m) if w is None else np.asarray(w, dtype=np.float64)
    assert wt.shape == (m,)
    keep_idx = np.zeros((B, n_keep - 1), dtype=np.int32)
    merged_idx = np.zeros((B, m), dtype=np.int32)
    for b in range(B):
        keep_idx[b], merged_idx[b] = partition(score_mean[b], n_keep)
    outs = []
    for plane, rule, dt in zip(planes, rules, dtypes):
        plane = np.asarray(plane)
        Bp, N, C = plane.shape
        assert Bp == B
        out = np.zeros((B, N - r, C), dtype=plane.dtype)
        for b in range(B):
            img = plane[b, img_begin:img_begin + n_img]
            if rule == RULE_WEIGHTED:
                p_new = wt @ img[merged_idx[b]].astype(np.float64)
                p_new = round_out(p_new, dt).astype(plane.dtype)
            else:
                p_new = img[merged_idx[b, 0]]
            out[b, :img_begin] = plane[b, :img_begin]
            out[b, img_begin:img_begin + n_keep - 1] = img[keep_idx[b]]
            out[b, img_begin + n_keep - 1] = p_new
            out[b, img_begin + n_keep:] = plane[b, img_begin + n_img:]
        outs.append(out)
    return outs, keep_idx, merged_idx


# --------------------------------------------------------------------------
# step 3b: similarity merge (named by the benchmark spec, NOT by the paper)
# --------------------------------------------------------------------------


def similarity_assign(hidden, score, n_keep: int):
    """Dominant set and nearest-dominant assignment of one row of tokens.

    hidden [n, C], score [n].  Dominant = the n_keep highest-scoring tokens, listed in ascending index
    (position p = 0..n_keep-1).  Every other token is assigned to the dominant token with the largest
    cosine similarity (ties: lower position).  Returns (dom_idx [n_keep], assign [n] = position of the
    dominant token each token ends up in (its own position for a dominant token), cos [n-n_keep, n_keep],
    rest_idx [n-n_keep] ascending).
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    n = hidden.shape[0]
    order = order_desc(score)
    dom = np.sort(order[:n_keep])
    rest = np.sort(order[n_keep:])
    norm = np.sqrt((hidden * hidden).sum(axis=1))
    norm = np.where(norm > 0, norm, 1.0)
    unit = hidden / norm[:, None]
    cos = unit[rest] @ unit[dom].T
    assign = np.zeros(n, dtype=np.int32)
    assign[dom] = np.arange(n_keep)
    if rest.size:
        assign[rest] = np.argmax(cos, axis=1)          # first maximum = lower position on ties
    return dom.astype(np.int32), assign, cos, rest.astype(np.int32)


def merge_similarity(hidden, size, score, n_keep: int, dtype: str = "f32"):
    """One row's similarity merge.  hidden [n, C], size [n], score [n].

    Each dominant token becomes the size-weighted mean of itself and the tokens assigned to it
    (similarity_assign), and sizes add.  Output in ascending original index.
    Returns (rows [n_keep, C], new_size [n_keep], dom_idx [n_keep], assign of the non-dominant tokens).
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    size = np.asarray(size, dtype=np.float64)
    dom, assign, _, rest = similarity_assign(hidden, score, n_keep)
    acc = np.zeros((n_keep, hidden.shape[1]), dtype=np.float64)
    tot = np.zeros(n_keep, dtype=np.float64)
    for t in range(hidden.shape[0]):                    # ascending token order
        acc[assign[t]] += size[t] * hidden[t]
        tot[assign[t]] += size[t]
    rows = round_out(acc / tot[:, None], dtype)
    return rows, tot.astype(np.float32), dom, assign[rest]


def merge_similar(planes, score_mean, *, img_begin: int, n_img: int, n_keep: int, size=None, rules=None,
                  dtypes=None, assign=None):
    """Similarity merge of a batch, every plane (this build's definition, not the paper's).

    planes[0] is the plane the similarity is measured on.  Output row order: rows before the image
    span, the n_keep dominant tokens in ascending original index (each replaced by its cluster's
    size-weighted mean on RULE_WEIGHTED planes, kept as is on RULE_TOP planes), rows after the span.
    size [B, n_img] (default all ones).  `assign` [B, n_img] overrides the nearest-dominant choice
    (used to check merged values under a given assignment).  n_keep == n_img changes nothing.
    Returns (out_planes, keep_idx [B,n_keep], assign [B,n_img], new_size [B,n_keep]).
    """
    score_mean = np.asarray(score_mean)
    B = score_mean.shape[0]
    r = n_img - n_keep
    rules = rules or [RULE_WEIGHTED] * len(planes)
    dtypes = dtypes or ["f32"] * len(planes)
    size = np.ones((B, n_img)) if size is None else np.asarray(size, dtype=np.float64)
    keep_idx = np.zeros((B, n_keep), dtype=np.int32)
    assign_out = np.zeros((B, n_img), dtype=np.int32)
    new_size = np.zeros((B, n_keep), dtype=np.float64)
    base = np.asarray(planes[0])
    for b in range(B):
        dom, a, _, _ = similarity_assign(base[b, img_begin:img_begin + n_img], score_mean[b], n_keep)
        if assign is not None:
            a = np.asarray(assign[b])
        keep_idx[b], assign_out[b] = dom, a
        np.add.at(new_size[b], a, size[b])
    outs = []
    for plane, rule, dt in zip(planes, rules, dtypes):
        plane = np.asarray(plane)
        N, C = plane.shape[1], plane.shape[2]
        out = np.zeros((B, N - r, C), dtype=plane.dtype)
        for b in range(B):
            img = plane[b, img_begin:img_begin + n_img]
            out[b, :img_begin] = plane[b, :img_begin]
            out[b, img_begin + n_keep:] = plane[b, img_begin + n_img:]
            if rule == RULE_WEIGHTED and r > 0:
                acc = np.zeros((n_keep, C), dtype=np.float64)
                for t in range(n_img):
                    acc[assign_out[b, t]] += size[b, t] * img[t].astype(np.float64)
                tot = np.where(new_size[b] > 0, new_size[b], 1.0)      # an empty cluster (imposed assignment only)
                out[b, img_begin:img_begin + n_keep] = round_out(acc / tot[:, None], dt).astype(plane.dtype)
            else:
                out[b, img_begin:img_begin + n_keep] = img[keep_idx[b]]
        outs.append(out)
    return outs, keep_idx, assign_out, new_size.astype(np.float32)


# --------------------------------------------------------------------------
# pyramid schedule   (App. A.2; Sec. 3.2.1 last par.)
# --------------------------------------------------------------------------


def schedule(n_img: int, final_keep: float, n_stages: int = 3):
    """Image-token count after each of the n_stages merge layers.

    App. A.2: a constant reduction ratio per stage, fixed by the budget.  With
    final keep fraction f the count after stage s is round-half-up of
    n_img * f^(s/S), always taken from the original n_img, never below 1.
    """
    out = []
    for s in range(1, n_stages + 1):
        v = int(math.floor(n_img * final_keep ** (s / n_stages) + 0.5))
        out.append(max(1, min(n_img, v)))
    return out


# --------------------------------------------------------------------------
# step 5: KV-cache compression   (Sec. 3.2.2; App. A.2: beta = 0.995)
# --------------------------------------------------------------------------

KIND_PROTECTED = 0   # system / instruction text
KIND_IMAGE = 1
KIND_GENERATED = 2

SCORE_FIX_SHIFT = 32          # fixed-point scale 2^32 for cumulative sums
SCORE_FIX_CLAMP = 65536.0     # scores are clamped to [0, 2^16] before scaling


def score_fixed_point(score) -> np.ndarray:
    """u = floor(clamp(score, 0, 2^16) * 2^32) as exact integers (NaN -> 0)."""
    s = np.asarray(score, dtype=np.float64)
    s = np.where(s > 0, s, 0.0)          # negatives and NaN -> 0
    s = np.minimum(s, SCORE_FIX_CLAMP)
    return np.floor(s * 4294967296.0).astype(np.uint64)


def kv_select_threshold(score, kind, length: int, beta: float) -> np.ndarray:
    """Keep mask over slots [0, length) of one (batch, KV head).

    Sec. 3.2.2: sort the image entries by score, highest first (A_des), and
    keep the shortest prefix whose accumulated score reaches beta times the
    total image score; drop the other image entries.  Sums are taken on the
    fixed-point integers above so the cut does not depend on summation order.
    Non-image entries are always kept.  beta >= 1 or a zero total keeps all.
    """
    score = np.asarray(score)[:length]
    kind = np.asarray(kind)[:length]
    keep = np.ones(length, dtype=bool)
    img = np.nonzero(kind == KIND_IMAGE)[0]
    if img.size == 0 or beta >= 1.0:
        return keep
    u = score_fixed_point(score[img])
    total = int(u.sum(dtype=np.uint64))
    if total == 0:
        return keep
    thresh = int(math.ceil(float(beta) * float(total)))
    order = order_desc(score[img])
    cum = 0
    n_kept = 0
    for o in order:
        cum += int(u[o])
        n_kept += 1
        if cum >= thresh:
            break
    keep[img[order[n_kept:]]] = False
    return keep


def kv_select_budget(score, kind, length: int, budget: int, n_recent: int) -> np.ndarray:
    """Keep mask for the fixed-budget eviction (this build's definition).

    Protected = text/system entries and the last n_recent slots.  Nothing
    happens while length <= budget.  Otherwise all protected entries stay and
    the budget is filled with the highest-scoring other entries (step-2
    order); with more protected entries than budget only they stay.
    """
    score = np.asarray(score)[:length]
    kind = np.asarray(kind)[:length]
    keep = np.ones(length, dtype=bool)
    if length <= budget:
        return keep
    slot = np.arange(length)
    protected = (kind == KIND_PROTECTED) | (slot >= length - n_recent)
    ev = np.nonzero(~protected)[0]
    room = max(0, budget - int(protected.sum()))
    order = order_desc(score[ev])
    keep[ev[order[room:]]] = False
    return keep


ORDER_STABLE = 0
ORDER_FILL = 1


def compaction_sources(keep, order: int) -> np.ndarray:
    """src[new_slot] = old slot that ends up there; len(src) = number kept.

    STABLE: survivors keep their ascending slot order.
    FILL: with n' survivors, a survivor in a slot < n' stays put; the i-th
    evicted slot below n' (ascending) receives the i-th survivor found at a
    slot >= n' (ascending).
    """
    keep = np.asarray(keep, dtype=bool)
    surv = np.nonzero(keep)[0]
    n_new = surv.size
    if order == ORDER_STABLE:
        return surv.astype(np.int64)
    src = np.arange(n_new, dtype=np.int64)
    holes = [s for s in range(n_new) if not keep[s]]
    tail = [s for s in range(n_new, keep.size) if keep[s]]
    assert len(holes) == len(tail)
    for h, t in zip(holes, tail):
        src[h] = t
    return src


def kv_compress(k_cache, v_cache, score, kind, orig_pos, length, *, mode: str,
                beta: float = 0.995, budget: int = 0, n_recent: int = 0,
                order: int = ORDER_STABLE):
    """Apply the eviction to every (batch, KV head); arrays are modified in a copy.

    k_cache, v_cache [B,Hkv,Lmax,d]; score f32, kind u8, orig_pos i32 [B,Hkv,Lmax];
    length [B,Hkv].  Slots at or beyond the new length keep whatever they held.
    Returns (k, v, score, kind, orig_pos, new_length, n_evicted).
    """
    k_cache, v_cache = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    score, kind = np.array(score, copy=True), np.array(kind, copy=True)
    orig_pos, length = np.array(orig_pos, copy=True), np.array(length, copy=True)
    B, Hkv = length.shape
    n_evicted = np.zeros_like(length)
    for b in range(B):
        for g in range(Hkv):
            L = int(length[b, g])
            if mode == "threshold":
                keep = kv_select_threshold(score[b, g], kind[b, g], L, beta)
            elif mode == "budget":
                keep = kv_select_budget(score[b, g], kind[b, g], L, budget, n_recent)
            else:
                raise ValueError(mode)
            src = compaction_sources(keep, order)
            n_new = src.size
            for arr in (k_cache, v_cache, score, kind, orig_pos):
                arr[b, g, :n_new] = arr[b, g, src]
            length[b, g] = n_new
            n_evicted[b, g] = L - n_new
    return k_cache, v_cache, score, kind, orig_pos, length, n_evicted


# --------------------------------------------------------------------------
# step 6: decode attention over the retained cache   (Sec. 3.2.2, par. 1)
# --------------------------------------------------------------------------


def decode_attn(q, k_new, v_new, k_cache, v_cache, score, kind, orig_pos, length, *,
                scale: float | None = None, score_decay: float = 1.0,
                new_kind: int = KIND_GENERATED, new_pos: int = 0,
                out_dtype: str = "f32", update_score: bool = True):
    """One decode step of every (batch, head) over its own retained entries.

    q [B,Hq,d]; k_new, v_new [B,Hkv,d] or None (no append).  The new entry is
    appended at slot length[b,g] with score 0, kind new_kind, position new_pos;
    the softmax then runs over slots [0, length) of the KV head the query head
    belongs to.  If update_score, each entry's importance continues the
    received-attention definition of Sec. 3.2.1 into decoding:
    score <- score_decay * score + mean over the G heads of the probabilities.
    Returns (out [B,Hq,d], k, v, score, kind, orig_pos, length) (copies).
    """
    q = np.asarray(q, dtype=np.float64)
    k_cache, v_cache = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    score, kind = np.array(score, copy=True), np.array(kind, copy=True)
    orig_pos, length = np.array(orig_pos, copy=True), np.array(length, copy=True)
    B, Hq, d = q.shape
    Hkv = k_cache.shape[1]
    G = Hq // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    scale = float(scale)
    decay = float(np.float32(score_decay))
    out = np.zeros((B, Hq, d), dtype=np.float64)
    for b in range(B):
        for g in range(Hkv):
            L = int(length[b, g])
            if k_new is not None:
                k_cache[b, g, L] = k_new[b, g]
                v_cache[b, g, L] = v_new[b, g]
                score[b, g, L] = 0.0
                kind[b, g, L] = new_kind
                orig_pos[b, g, L] = new_pos
                L += 1
                length[b, g] = L
            if L == 0:
                continue
            kk = np.asarray(k_cache[b, g, :L], dtype=np.float64)
            vv = np.asarray(v_cache[b, g, :L], dtype=np.float64)
            p_sum = np.zeros(L, dtype=np.float64)
            for h in range(g * G, (g + 1) * G):
                s = scale * (kk @ q[b, h])
                e = np.exp(s - s.max())
                p = e / e.sum()
                out[b, h] = p @ vv
                p_sum += p
            if update_score:
                new = decay * np.asarray(score[b, g, :L], dtype=np.float64) + p_sum / G
                score[b, g, :L] = new.astype(np.float32)
    return round_out(out, out_dtype), k_cache, v_cache, score, kind, orig_pos, length
