"""The synthetic workloads against what the paper prints about its own inputs (CPU; oracle only)."""
import json
import os

import numpy as np

from oracle import lvlm_oracle as O
from workloads import configs, synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _tokens_for(score, frac):
    a = np.sort(np.asarray(score, dtype=np.float64))[::-1]
    return int(np.searchsorted(np.cumsum(a) / a.sum(), frac) + 1)


def test_attention_concentration_follows_the_pilot_study_and_grows_with_depth():
    """Sec. 3.1 (Fig. 2b): at layer 1, 188 of 1476 image tokens hold 95 % of the image attention; at layer 27, 49
    hold 90 % and 107 hold 95 %.  The pilot-shaped workload must reproduce these counts (they fix its one
    parameter per end of the stack), concentration must grow with depth, and with it the threshold rule of Sec. 3.2.2
    at the paper's beta = 0.995 must keep fewer entries per head the deeper the layer."""
    with open(os.path.join(GOLDEN, "paper_constants.json")) as f:
        gold = json.load(f)["attention_concentration"]
    w = configs.CFG7
    assert w.n_img == gold["layer1"]["n_img"] == gold["layer27"]["n_img"] and w.layers == 28
    kept, need95 = [], []
    for layer in (1, 9, 18, 27):
        x = synth.layer_inputs(w, layer=layer, with_v=False)
        sh, sm = O.score_tokens(x["q"].double().numpy(), x["k"].double().numpy(), q_pos0=w.n_sys + w.n_img,
                                img_begin=w.n_sys, n_img=w.n_img)
        need95.append(_tokens_for(sm[0], 0.95))
        if layer == 1:
            assert abs(need95[-1] - gold["layer1"]["tokens_for_95pct"]) <= 12
        if layer == 27:
            assert abs(_tokens_for(sm[0], 0.90) - gold["layer27"]["tokens_for_90pct"]) <= 6
            assert abs(need95[-1] - gold["layer27"]["tokens_for_95pct"]) <= 12
        kind = np.ones(w.n_img, dtype=np.uint8)
        kept.append(sum(int(O.kv_select_threshold(sh[0, h], kind, w.n_img, gold_beta()).sum()) for h in range(w.n_kv_heads)))
    assert need95[0] > need95[1] > need95[2] > need95[3]
    assert kept[0] > kept[1] > kept[2] > kept[3]            # one beta: shallow layers keep more, deep layers fewer


def gold_beta():
    with open(os.path.join(GOLDEN, "paper_constants.json")) as f:
        return json.load(f)["kv_beta"]


def test_decode_stream_draws_in_bulk_follow_the_same_law():
    # many(n) continues the running mean and returns n steps of the documented shapes
    w = configs.CFG4
    s = synth.DecodeStream(w)
    q, k, v = s.many(50)
    assert q.shape == (50, w.batch, w.n_q_heads, w.head_dim) and k.shape == v.shape == (50, w.batch, w.n_kv_heads, w.head_dim)
    drift = s.mean.float().std().item()
    assert 0.03 < drift < 0.12                                # 50 steps of sigma 0.01: about 0.07
    q1, k1, v1 = s.next()
    assert q1.shape == (w.batch, w.n_q_heads, w.head_dim)
    assert abs(k.float().std().item() - 1.0) < 0.05 and abs(v.float().std().item() - 1.0) < 0.05
