"""Long decode runs of configurations 4 and 5 against the oracle (Sec. 3.2.2 carried through thousands of steps).

Every generated token appends an entry, attends over the retained entries, updates every entry's importance
(score <- 0.9 score + mean probability: the received-attention score of Sec. 3.2.1 continued into decoding) and,
once a head is at its budget, evicts one entry -- all inside lvlm_decode_attn, at the shapes and with the launch
arguments bench.py uses.  A CPU replay of the whole run would take hours, so the protocol is:
  * the first 64 steps: every step is checked against the oracle applied to the GPU's state just before it
    (attention output and importance within tolerance; appended entry, evicted entry, slot moves and lengths
    exact, the eviction decided by the oracle on the GPU's own score bits), and beside it the oracle runs FREE
    from its own previous state: wherever its kept set departs from the GPU's, the two entries in question must
    be a near-tie in the oracle's own scores (within 1e-5 of the largest score), after which the oracle takes the
    GPU's state of that head and goes on;
  * after that: the same single-step check from copied-back GPU state at every 256th step and at the last one.
The GPU always runs the full batch; the oracle looks at a sample of (sequence, KV head) pairs per checked step
and at all of them at the first and the last step.
"""
import os
import sys

import numpy as np
import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402
import paper_2509_00419_amd as lv  # noqa: E402
from oracle import lvlm_oracle as O  # noqa: E402
from workloads import configs, synth  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DECAY = 0.9


def f64(t):
    return t.detach().double().cpu().numpy()


def rel_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def head_state(state, b, g):
    """Host copy of one (sequence, KV head) pair of a cache [k, v, score, kind, pos, len], shaped [1, 1, ...]."""
    k, v, score, kind, pos, length = state
    return [f64(k[b:b + 1, g:g + 1]), f64(v[b:b + 1, g:g + 1]), score[b:b + 1, g:g + 1].cpu().numpy().copy(),
            kind[b:b + 1, g:g + 1].cpu().numpy().copy(), pos[b:b + 1, g:g + 1].cpu().numpy().copy(),
            length[b:b + 1, g:g + 1].cpu().numpy().copy()]


def same_head(now, ref, exact_score, what):
    assert np.array_equal(now[5], ref[5]), what
    n = int(now[5][0, 0])
    for i in (0, 1, 3, 4):
        assert np.array_equal(now[i][0, 0, :n], ref[i][0, 0, :n]), (what, i)
    if exact_score:
        assert np.array_equal(now[2][0, 0, :n], ref[2][0, 0, :n]), what
    elif n:
        assert rel_err(now[2][0, 0, :n], ref[2][0, 0, :n]) < 1e-5, what


def run_long_decode(ctx, w, state, stream, n_steps, pos0, sample, tol=2e-2, first=64, every=256):
    """state: device [k, v, score, kind, pos, len] of one layer; stream: its DecodeStream.  Returns counters."""
    B, H, G, budget = w.batch, w.n_kv_heads, w.group, w.kv_budget
    all_heads = [(b, g) for b in range(B) for g in range(H)]
    free = {}                                   # (b, g) -> the free-running oracle's state of that head
    stats = {"checked": 0, "evictions": 0, "free_departures": 0}
    chunk = 256
    for t0 in range(0, n_steps, chunk):
        n = min(chunk, n_steps - t0)
        qs, ks, vs = stream.many(n)
        for j in range(n):
            t = t0 + j
            q, kn, vn = qs[j], ks[j], vs[j]
            checked = t < first or t % every == 0 or t == n_steps - 1
            heads = all_heads if t in (0, n_steps - 1) else sample
            kw = dict(score_decay=DECAY, new_pos=pos0 + t, len_bound=budget + 1)
            if checked:
                before = {h: head_state(state, *h) for h in heads}
                cp = [x.clone() for x in state]
                plain = ctx.decode_attn(q, kn, vn, *cp, **kw)                 # the GPU's score bits before eviction
            out = ctx.decode_attn(q, kn, vn, *state, evict_budget=budget, evict_recent=1, **kw)
            if not checked:
                continue
            torch.cuda.synchronize()
            assert torch.equal(out, plain), t
            stats["checked"] += 1
            qh, kh, vh = f64(q), f64(kn), f64(vn)
            for (b, g) in heads:
                what = (t, b, g)
                q1, k1, v1 = qh[b:b + 1, g * G:(g + 1) * G], kh[b:b + 1, g:g + 1], vh[b:b + 1, g:g + 1]
                ref = O.decode_attn(q1, k1, v1, *before[(b, g)], score_decay=DECAY, new_pos=pos0 + t, out_dtype=w.dtype)
                assert rel_err(f64(out[b, g * G:(g + 1) * G]), ref[0][0]) < tol, what
                mid = head_state(cp, b, g)
                same_head(mid, list(ref[1:]), False, what)
                ref2 = O.kv_compress(*mid, mode="budget", budget=budget, n_recent=1, order=O.ORDER_FILL)
                now = head_state(state, b, g)
                same_head(now, list(ref2[:6]), True, what)
                stats["evictions"] += int(ref2[6][0, 0])
                assert int(now[5][0, 0]) <= budget
                # ---- the oracle running free beside the GPU (first steps only)
                if t < first and (b, g) in sample:
                    if (b, g) not in free:
                        free[(b, g)] = before[(b, g)]
                    fr = O.decode_attn(q1, k1, v1, *free[(b, g)], score_decay=DECAY, new_pos=pos0 + t, out_dtype=w.dtype)
                    fr2 = O.kv_compress(*fr[1:], mode="budget", budget=budget, n_recent=1, order=O.ORDER_FILL)
                    n_now = int(now[5][0, 0])
                    if np.array_equal(fr2[5], now[5]) and np.array_equal(fr2[4][0, 0, :n_now], now[4][0, 0, :n_now]):
                        assert rel_err(f64(out[b, g * G:(g + 1) * G]), fr[0][0]) < tol, what
                        assert rel_err(now[2][0, 0, :n_now], fr2[2][0, 0, :n_now]) < 1e-4, what
                        free[(b, g)] = list(fr2[:6])
                    else:
                        # the kept sets part: the entry the GPU evicted and the one the oracle evicted must be a
                        # near-tie in the oracle's own scores
                        stats["free_departures"] += 1
                        n_mid = int(fr[6][0, 0])
                        pos_mid, sc_mid = fr[5][0, 0, :n_mid], fr[3][0, 0, :n_mid].astype(np.float64)
                        gone_gpu = np.setdiff1d(pos_mid, now[4][0, 0, :n_now])
                        gone_orc = np.setdiff1d(pos_mid, fr2[4][0, 0, :int(fr2[5][0, 0])])
                        assert gone_gpu.size == 1 and gone_orc.size == 1, what
                        s_gpu = sc_mid[pos_mid == gone_gpu[0]][0]
                        s_orc = sc_mid[pos_mid == gone_orc[0]][0]
                        assert abs(s_gpu - s_orc) <= 1e-5 * np.abs(sc_mid).max(), (what, s_gpu, s_orc)
                        free[(b, g)] = now
    return stats


def test_config4_long_decode():
    """Config 4: B = 16, 28 / 4 heads, prefill of 1024 tokens (64 system + 768 image + 192 instruction), budget 1024
    per KV head, 4096 generated tokens whose queries and keys follow a slowly drifting mean, eviction every step."""
    w = configs.CFG4
    ctx = lv.Context(0)
    x = synth.layer_inputs(w, layer=0, device=DEV)
    B, H, d, N = w.batch, w.n_kv_heads, w.head_dim, w.seq_len
    assert N == w.kv_budget
    Lmax = w.kv_budget + 8
    k = torch.zeros(B, H, Lmax, d, dtype=torch.bfloat16, device=DEV)
    v = torch.zeros_like(k)
    k[:, :, :N] = x["k"].permute(0, 2, 1, 3)
    v[:, :, :N] = x["v"].permute(0, 2, 1, 3)
    score = torch.zeros(B, H, Lmax, device=DEV)
    ctx.score_tokens(x["q"], x["k"], q_pos0=w.n_sys + w.n_img, img_begin=w.n_sys, n_img=w.n_img,
                     score_head=score[:, :, w.n_sys:w.n_sys + w.n_img])        # prefill importance of the image entries
    kind = torch.zeros(B, H, Lmax, dtype=torch.uint8, device=DEV)
    kind[:, :, w.n_sys:w.n_sys + w.n_img] = lv.KIND_IMAGE
    pos = torch.arange(Lmax, dtype=torch.int32, device=DEV).view(1, 1, Lmax).expand(B, H, Lmax).contiguous()
    length = torch.full((B, H), N, dtype=torch.int32, device=DEV)
    state = [k, v, score, kind, pos, length]
    sample = [(0, 0), (3, 1), (7, 2), (15, 3), (9, 0), (12, 2)]
    stats = run_long_decode(ctx, w, state, synth.DecodeStream(w, layer=0, device=DEV), w.decode_steps, N, sample)
    torch.cuda.synchronize()
    assert stats["checked"] == 64 + 15 + 1 and stats["evictions"] > 0
    assert int(length.min()) == w.kv_budget == int(length.max())
    # after 4096 steps the caches hold generated entries as well as image entries; every protected entry is there
    assert int((kind[:, :, :N] == lv.KIND_PROTECTED).sum()) == B * H * (w.n_sys + w.n_text)
    assert int((kind[:, :, :N] == lv.KIND_GENERATED).sum()) > 0
    print(f"[long decode cfg4] {stats}")


def test_config5_long_decode_two_layers():
    """Config 5: layer 0 (16512 entries cut to the 2048 budget before generation) and the last layer (what the pyramid
    and the threshold rule leave of 620 entries, some 260: it grows until it reaches the budget, then evicts), 2048 generated tokens."""
    w = configs.CFG5
    ctx = lv.Context(0)
    layers = bench.plan(w, lv)
    master = bench.build_master(w, layers, torch, synth, DEV)
    st = bench.StepState(w, layers, master, torch, prefill_order="fill")
    bench.run_prefill(ctx, lv, w, st, reserve=True)
    torch.cuda.synchronize()
    del master
    B, L = w.batch, w.kv_budget + 8
    for li in (0, len(layers) - 1):
        sl = slice(li * B, (li + 1) * B)
        state = [st.k[sl, :, :L].contiguous(), st.v[sl, :, :L].contiguous(), st.score[sl, :, :L].contiguous(),
                 st.kind[sl, :, :L].contiguous(), st.pos[sl, :, :L].contiguous(), st.len[sl].clone()]
        start = int(state[5].min())
        assert (start == w.kv_budget) if li == 0 else (128 < start < 700)
        sample = [(0, 0), (0, 3), (0, 7)]
        stats = run_long_decode(ctx, w, state, synth.DecodeStream(w, layer=li, device=DEV), w.decode_steps, w.seq_len,
                                sample)
        torch.cuda.synchronize()
        assert stats["checked"] == 64 + 7 + 1
        assert int(state[5].min()) == w.kv_budget == int(state[5].max())
        assert int((state[3][:, :, :w.kv_budget] == lv.KIND_PROTECTED).sum()) == B * w.n_kv_heads * w.n_text
        assert stats["evictions"] > 0
        print(f"[long decode cfg5 layer {li}] {stats}")
