#!/usr/bin/env python3
"""Benchmark of the LightVLM token-reduction path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch.  The default workload is config 5, the
largest single-GPU shape (InternVL2.5-26B-like stack: 48 layers, 16384 image + 128 instruction tokens, bf16,
48 / 8 heads); --workload selects the others.

  prefill, decoder layers l >= the first compressed layer:  lvlm_score_tokens (instruction queries x all keys
      of a layer, written straight into that layer's cache scores), issued once per run of layers with the
      same token count -- at the pyramid layer that ends the run, which needs its score for the merge, with
      the run's layers stacked along the batch axis;
      at the pyramid layers: lvlm_merge_compact of the hidden states and position ids;
  after the last layer: ONE lvlm_kv_compress (threshold beta = 0.995) over the per-head caches of all compressed
      layers, then, where the workload has a per-head budget, ONE lvlm_kv_compress (fixed budget) that brings
      every cache of every layer down to it "before generation" (Sec. 3.2.2);
  decode, one generated token in STEADY STATE: per layer lvlm_decode_attn on a cache that holds exactly `budget`
      entries: append + GQA attention over the retained entries + importance update + eviction of one entry,
      all in the one call.  Where prefill leaves some layers short of the budget (config 5: the deep layers
      hold 620 entries) the steady-state caches are made during set-up by running the path itself forward --
      decode steps with eviction -- until every layer is full.  The first decode step right after prefill is
      timed as well and reported under its own name.  Workloads whose budget never binds decode over the caches
      as prefill left them.

Inputs are resident in HBM before the timed region.  Every step works on its own copy of the state (caches are
modified in place), so no step re-reads buffers a previous step left in cache.  Each step is a pair of HIP graphs
(prefill, decode) captured beforehand; the timed region replays them.

Prints ONE JSON line: metric, value (image tokens/s over the whole step), ms_per_step, decode steps/s of the
steady state, the roofline of the dominant kernel (the one with the most time per step among ALL kernels of the
path; algorithmic bytes or flops over its measured launch time), the CPU oracle timed beside it, per-kernel rows.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_F32_PEAK_TFLOPS = 157.3


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg6"],
                    help="cfg5 (default): the largest single-GPU configuration; cfg2 is a latency row only")
    ap.add_argument("--row-lse", default="computed", choices=["computed", "given"],
                    help="row normalisers of the scoring step: computed by the library (default: one more pass over "
                         "the keys) or given, as a prefill attention kernel that emits its log-sum-exp would (Sec. "
                         "3.2.1: the scores then cost one pass over the image keys)")
    ap.add_argument("--prefill-order", default="fill", choices=["stable", "fill"],
                    help="slot order after the compression of the caches at the end of prefill: holes filled from "
                         "the tail (fill, default: only as many entries move as were evicted; attention needs no "
                         "slot order) or survivors in ascending slot order (stable: rewrites almost the whole cache)")
    ap.add_argument("--per-layer", action="store_true",
                    help="one score / compression call per layer instead of one per run of layers / per step "
                         "(the launch sequence of a caller that batches nothing); default: batched")
    ap.add_argument("--merge", default="rank", choices=["rank", "similar"],
                    help="merge rule at the pyramid layers: the paper's rank weights (lvlm_merge_compact) or the "
                         "similarity merge (lvlm_merge_similar)")
    ap.add_argument("--op", default="step", choices=["step", "prefill_attn", "stream", "score_load"],
                    help="step: the token-reduction path (the default, the headline metric); prefill_attn: "
                         "lvlm_prefill_attn alone over the layer stack -- the layers' own attention at the token "
                         "counts the pyramid leaves, with the scores as its by-product where the path scores; "
                         "stream: lvlm_stream_probe over buffers of the size of one decode layer's K and V rows -- what "
                         "a launch of that size can stream at all, by workgroup count; score_load: lvlm_score_tokens "
                         "alone at the workload's scoring shapes for 4 to 32 sequences per call -- how the time of the "
                         "one-launch score kernel steps with the workgroups per compute unit")
    ap.add_argument("--decode-evict", choices=["batched", "fused"], default="batched",
                    help="steady-state decode: one lvlm_kv_compress over all layers' caches at the end of the step "
                         "(batched), or the eviction inside every layer's lvlm_decode_attn call (fused)")
    ap.add_argument("--profile-steps", type=int, default=3, help="eager steps timed per kernel with HIP events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (a reference of known traffic for rocprofv3 --pmc)")
    return ap.parse_args()


# ----------------------------------------------------------------------------- workload plan
def plan(w, lv):
    """Per-layer image-token counts and which calls run where (host arithmetic only)."""
    if w.name.startswith("cfg2"):
        # "keep fraction falls 100 % -> 35 % -> 3 % across the pyramid layers": explicit counts
        keeps = [int(w.n_img * f + 0.5) for f in (1.0, 0.35, 0.03)]
    elif w.merge_layers:
        keeps = lv.schedule(w.n_img, w.final_keep[-1], len(w.merge_layers))
    else:
        keeps = []
    layers = []
    n_img = w.n_img
    for l in range(w.layers):
        entry = {"layer": l, "n_img": n_img, "score": bool(w.merge_layers) and l >= w.kv_first_layer,
                 "merge_to": None, "kv_threshold": bool(w.merge_layers) and l >= w.kv_first_layer}
        if l in w.merge_layers:
            entry["merge_to"] = keeps[w.merge_layers.index(l)]
        layers.append(entry)
        if entry["merge_to"] is not None:
            n_img = entry["merge_to"]
    return layers


def score_groups(layers, per_layer=False):
    """Runs of consecutive scored layers with the same image-token count, as (first, last) layer indices.  A
    run ends at a layer that really merges (it needs its score at once) or with the stack; the layers before it
    in the run feed only the cache compression after prefill, so one call at the run's end scores them all: their
    instruction-token queries [T,Hq,d] and their caches are kept until then."""
    groups, first = [], None
    for i, en in enumerate(layers):
        if not en["score"]:
            assert first is None
            continue
        if first is None:
            first = i
        merges = en["merge_to"] is not None and en["merge_to"] < en["n_img"]      # a 100 % stage merges nothing
        if per_layer or merges or i + 1 == len(layers) or not layers[i + 1]["score"] \
                or layers[i + 1]["n_img"] != en["n_img"]:
            groups.append((first, i))
            first = None
    return groups


EXTRA_SLOTS = 8     # free cache slots per head beyond the prefill length


def cache_slots(w):
    """Slots per head of every layer's cache (all layers alike, so that their caches stack into one tensor)."""
    return w.n_sys + w.n_img + w.n_text + EXTRA_SLOTS


class StepState:
    """Device buffers of one step: the KV caches of all layers live in ONE tensor [layers*B, H, Lmax, d] (and
    likewise scores, kinds, positions, lengths), so that one lvlm_kv_compress call can serve many layers;
    every layer works on its own [B, ...] slice."""

    def __init__(self, w, layers, master, torch, per_layer=False, prefill_order="stable", given_lse=False):
        self.per_layer = per_layer      # one call per layer instead of one per run of layers / per step
        self.prefill_order = prefill_order
        B, H, d, L = w.batch, w.n_kv_heads, w.head_dim, cache_slots(w)
        dev, dt = master[0]["k"].device, master[0]["k"].dtype
        nl = len(layers)
        self.k = torch.empty(nl * B, H, L, d, dtype=dt, device=dev)
        self.v = torch.empty(nl * B, H, L, d, dtype=dt, device=dev)
        self.score = torch.empty(nl * B, H, L, dtype=torch.float32, device=dev)
        self.kind = torch.empty(nl * B, H, L, dtype=torch.uint8, device=dev)
        self.pos = torch.empty(nl * B, H, L, dtype=torch.int32, device=dev)
        self.len = torch.empty(nl * B, H, dtype=torch.int32, device=dev)
        self.n_evicted = torch.empty(nl * B, H, dtype=torch.int32, device=dev)
        self.q = torch.empty(nl * B, w.n_text, w.n_q_heads, d, dtype=dt, device=dev)     # instruction-token queries
        # natural-log sum-exp of every instruction row's scaled logits, as an attention kernel would leave it
        self.row_lse = None
        if given_lse:
            self.row_lse = torch.zeros(nl * B, w.n_q_heads, w.n_text, dtype=torch.float32, device=dev)
            for i, m in enumerate(master):
                if "row_lse" in m:
                    self.row_lse[i * B:(i + 1) * B] = m["row_lse"]
        self.groups = score_groups(layers, per_layer)
        # head-mean scores [g*B, n_img] of each group; the merge reads the last layer's rows
        self.group_mean = {last: torch.empty((last - first + 1) * B, layers[last]["n_img"], dtype=torch.float32,
                                             device=dev) for first, last in self.groups}
        self.group_first = {last: first for first, last in self.groups}
        self.layers = [LayerState(w, en, master, torch, self, i) for i, en in enumerate(layers)]
        # the layers whose cache the threshold rule compresses after prefill: a contiguous tail of the stack
        first = [i for i, en in enumerate(layers) if en["kv_threshold"]]
        self.kv_from = first[0] * B if first else None
        assert not first or first == list(range(first[0], nl)), "compressed layers must be the last ones"
        self.kv_bound = max((st.N for st in self.layers[first[0]:]), default=0) if first else 0
        self.all_bound = max(st.N for st in self.layers)
        # most entries a head can hold at its first decode step: what prefill leaves (cut to the budget) plus one
        self.dec_bound = max(st.dec_bound for st in self.layers)

    def tail(self, t):
        return t[self.kv_from:]

    def __iter__(self):
        return iter(self.layers)

    def __getitem__(self, i):
        return self.layers[i]


class LayerState:
    """Views and buffers of one decoder layer for one step."""

    def __init__(self, w, entry, master, torch, step, index):
        B, H, d = w.batch, w.n_kv_heads, w.head_dim
        self.entry = entry
        self.n_img = entry["n_img"]
        self.N = w.n_sys + self.n_img + w.n_text
        self.Lmax = cache_slots(w)
        self.dec_bound = min(self.Lmax, (min(self.N, w.kv_budget) if w.kv_budget > 0 else self.N) + 1)
        m = master[entry["layer"]]
        sl = slice(index * B, (index + 1) * B)
        self.q = step.q[sl]                                       # [B,T,Hq,d]
        self.q.copy_(m["q"])
        self.k, self.v = step.k[sl], step.v[sl]                   # [B,H,Lmax,d] head-major cache (slice of the stack)
        self.score, self.kind, self.pos, self.len = step.score[sl], step.kind[sl], step.pos[sl], step.len[sl]
        self.n_evicted = step.n_evicted[sl]
        for dst, name in ((self.k, "k"), (self.v, "v"), (self.score, "score"), (self.kind, "kind"), (self.pos, "pos"),
                          (self.len, "len")):
            dst.copy_(m[name])
        self.hidden = m["hidden"].clone() if "hidden" in m else None
        self.pos_ids = m["pos_ids"].clone() if "pos_ids" in m else None
        # head-mean scores: the last B rows of the group's array when this layer ends a scoring group
        self.score_mean = step.group_mean[index][-B:] if index in step.group_mean else None
        if entry["merge_to"] is not None:
            r = self.n_img - entry["merge_to"]
            self.hidden_out = torch.empty(B, self.N - r, w.hidden, dtype=self.hidden.dtype, device=self.q.device)
            self.pos_out = torch.empty(B, self.N - r, 3, dtype=torch.int32, device=self.q.device)
            self.keep_idx = torch.empty(B, max(entry["merge_to"] - 1, 1), dtype=torch.int32, device=self.q.device)
            self.merged_idx = torch.empty(B, r + 1, dtype=torch.int32, device=self.q.device)
            # similarity merge: all n_keep dominant tokens are listed, every image token gets an assignment
            self.dom_idx = torch.empty(B, entry["merge_to"], dtype=torch.int32, device=self.q.device)
            self.assign = torch.empty(B, self.n_img, dtype=torch.int32, device=self.q.device)
            self.size_out = torch.empty(B, entry["merge_to"], dtype=torch.float32, device=self.q.device)
        self.q_dec = m["q_dec"].clone()
        self.k_dec = m["k_dec"].clone()
        self.v_dec = m["v_dec"].clone()
        self.out_dec = torch.empty_like(self.q_dec)


class SteadyLayer:
    """One layer's cache in steady-state decode (exactly `budget` entries per head), with its decode inputs."""

    def __init__(self, w, sl, step, src, torch):
        self.k, self.v, self.score, self.kind, self.pos, self.len = (step.k[sl], step.v[sl], step.score[sl],
                                                                     step.kind[sl], step.pos[sl], step.len[sl])
        self.Lmax = step.k.shape[2]
        self.dec_bound = w.kv_budget + 1
        self.q_dec, self.k_dec, self.v_dec = src.q_dec.clone(), src.k_dec.clone(), src.v_dec.clone()
        self.out_dec = torch.empty_like(self.q_dec)


class SteadyState:
    """The caches of all layers in steady-state decode, stacked like StepState's: [layers*B, H, budget + 8, d].
    Made from a state that went through prefill by running the path itself forward (decode steps that append and
    evict) until every head of every layer holds `budget` entries; clone() copies it for the other steps."""

    def __init__(self, w, torch, template):
        self.per_layer = False
        self.prefill_order = "fill"
        self.w = w
        t = template
        self.k, self.v = torch.empty_like(t.k), torch.empty_like(t.v)
        self.score, self.kind = torch.empty_like(t.score), torch.empty_like(t.kind)
        self.pos, self.len = torch.empty_like(t.pos), torch.empty_like(t.len)
        for name in ("k", "v", "score", "kind", "pos", "len"):
            getattr(self, name).copy_(getattr(t, name))
        B = w.batch
        self.layers = [SteadyLayer(w, slice(i * B, (i + 1) * B), self, src, torch) for i, src in enumerate(t.layers)]
        self.dec_bound = w.kv_budget + 1
        self.steps_run = getattr(t, "steps_run", 0)

    @classmethod
    def from_prefilled(cls, w, torch, synth, ctx, lv, st):
        """st: a StepState after run_prefill.  Copies its (already budget-sized) caches into compact tensors and
        decodes forward, one generated token at a time over all layers, until no head is short of the budget."""
        B, H, d, L = w.batch, w.n_kv_heads, w.head_dim, w.kv_budget + EXTRA_SLOTS
        nl = len(st.layers)

        class _T:
            pass
        t = _T()
        t.k, t.v = st.k[:, :, :L].contiguous(), st.v[:, :, :L].contiguous()
        t.score, t.kind, t.pos = st.score[:, :, :L].contiguous(), st.kind[:, :, :L].contiguous(), st.pos[:, :, :L].contiguous()
        t.len = st.len.clone()
        t.layers = st.layers
        assert int(t.len.max()) <= w.kv_budget
        self = cls(w, torch, t)
        n_fill = w.kv_budget - int(self.len.min())
        streams = [synth.DecodeStream(w, layer=st.layers[i].entry["layer"], device=self.k.device) for i in range(nl)]
        for s in streams:
            s.next()                                     # the draw the first decode step after prefill uses
        chunk = 256
        for t0 in range(0, n_fill, chunk):
            n = min(chunk, n_fill - t0)
            draws = [s.many(n) for s in streams]
            print(f"[bench] steady-state caches: decode step {t0} of {n_fill}", file=sys.stderr, flush=True)
            for j in range(n):
                for i, L_ in enumerate(self.layers):
                    q, k, v = draws[i]
                    ctx.decode_attn(q[j], k[j], v[j], L_.k, L_.v, L_.score, L_.kind, L_.pos, L_.len, score_decay=0.9,
                                    new_pos=w.seq_len + 1 + t0 + j, len_bound=w.kv_budget + 1, out=L_.out_dec,
                                    evict_budget=w.kv_budget, evict_recent=1, reserve=(t0 == 0 and j == 0))
                if j % 16 == 15:
                    torch.cuda.synchronize()         # keeps the launch queue short (a counter-collecting profiler has
                                                     # crashed on a queue some ten thousand launches deep)
        for i, L_ in enumerate(self.layers):             # the inputs of the timed step: the stream's next draw
            q, k, v = streams[i].next()
            L_.q_dec.copy_(q); L_.k_dec.copy_(k); L_.v_dec.copy_(v)
        torch.cuda.synchronize()
        assert int(self.len.min()) == w.kv_budget and int(self.len.max()) == w.kv_budget
        self.steps_run = n_fill
        return self

    def clone(self, torch):
        return SteadyState(self.w, torch, self)

    def __iter__(self):
        return iter(self.layers)

    def __getitem__(self, i):
        return self.layers[i]


def row_lse_of(q, k, q_pos0, torch):
    """[B,Hq,T] natural-log sum-exp over the causally visible keys of q.k / sqrt(d) (fp32, plain torch: set-up)."""
    B, T, Hq, d = q.shape
    N, Hkv = k.shape[1], k.shape[2]
    out = torch.empty(B, Hq, T, dtype=torch.float32, device=q.device)
    vis = torch.arange(N, device=q.device)[None, :] <= (q_pos0 + torch.arange(T, device=q.device))[:, None]
    for h in range(Hq):
        s = torch.einsum("btd,bnd->btn", q[:, :, h].float(), k[:, :, h // (Hq // Hkv)].float()) / math.sqrt(d)
        out[:, h] = torch.logsumexp(s.masked_fill(~vis, float("-inf")), dim=-1)
    return out


def build_master(w, layers, torch, synth, dev, given_lse=False):
    """One set of inputs per layer, generated on the GPU (seeded)."""
    master = []
    B, H, d = w.batch, w.n_kv_heads, w.head_dim
    for entry in layers:
        l, n_img = entry["layer"], entry["n_img"]
        x = synth.layer_inputs(w, layer=l, n_img=n_img, device=dev)
        N = x["k"].shape[1]
        Lmax = cache_slots(w)
        m = {"q": x["q"]}
        if given_lse and entry["score"]:
            m["row_lse"] = row_lse_of(x["q"], x["k"], w.n_sys + n_img, torch)
        for name in ("k", "v"):
            cache = torch.zeros(B, H, Lmax, d, dtype=x[name].dtype, device=dev)
            cache[:, :, :N] = x[name].permute(0, 2, 1, 3)
            m[name] = cache
        m["score"] = torch.zeros(B, H, Lmax, dtype=torch.float32, device=dev)
        kind = torch.zeros(B, H, Lmax, dtype=torch.uint8, device=dev)
        kind[:, :, w.n_sys:w.n_sys + n_img] = 1
        m["kind"] = kind
        m["pos"] = torch.arange(Lmax, dtype=torch.int32, device=dev).view(1, 1, Lmax).expand(B, H, Lmax).contiguous()
        m["len"] = torch.full((B, H), N, dtype=torch.int32, device=dev)
        if entry["merge_to"] is not None:
            m["hidden"] = x["hidden"]
            m["pos_ids"] = x["pos"].expand(B, N, 3).contiguous()
        stream = synth.DecodeStream(w, layer=l, device=dev)
        m["q_dec"], m["k_dec"], m["v_dec"] = stream.next()
        master.append(m)
    return master


def run_prefill(ctx, lv, w, states, reserve, merge="rank"):
    run_prefill_layers(ctx, lv, w, states, reserve, merge)
    run_prefill_compress(ctx, lv, w, states, reserve)
    run_prefill_budget(ctx, lv, w, states, reserve)


def run_prefill_layers(ctx, lv, w, states, reserve, merge="rank"):
    """Scoring and merging, in layer order."""
    B = w.batch
    for i, st in enumerate(states):
        e = st.entry
        img0 = w.n_sys
        if i in states.group_first:
            # one call scores every layer of the group that ends here (layers stacked along the batch axis)
            sl = slice(states.group_first[i] * B, (i + 1) * B)
            k_view = states.k[sl, :, :st.N].permute(0, 2, 1, 3)     # [g*B,N,H,d] view of the head-major caches
            sh_view = states.score[sl, :, img0:img0 + st.n_img]     # scores land in the caches' score arrays
            ctx.score_tokens(states.q[sl], k_view, q_pos0=img0 + st.n_img, img_begin=img0, n_img=st.n_img,
                             row_lse=None if states.row_lse is None else states.row_lse[sl],
                             score_head=sh_view, score_mean=states.group_mean[i], reserve=reserve)
        if e["merge_to"] is not None and merge == "similar":
            ctx.merge_similar([st.hidden, st.pos_ids], st.score_mean, img_begin=img0, n_img=st.n_img,
                              n_keep=e["merge_to"], rules=[lv.RULE_WEIGHTED, lv.RULE_TOP],
                              outs=[st.hidden_out, st.pos_out], keep_idx=st.dom_idx, assign=st.assign,
                              size_out=st.size_out, reserve=reserve)
        elif e["merge_to"] is not None:
            ctx.merge_compact([st.hidden, st.pos_ids], st.score_mean, img_begin=img0, n_img=st.n_img,
                              n_keep=e["merge_to"], rules=[lv.RULE_WEIGHTED, lv.RULE_TOP],
                              outs=[st.hidden_out, st.pos_out], keep_idx=st.keep_idx, merged_idx=st.merged_idx,
                              reserve=reserve)


def run_prefill_compress(ctx, lv, w, states, reserve):
    # survivors keep their slot order (stable) or the holes are filled from the tail (fill: moves only as many
    # entries as were evicted)
    order = lv.ORDER_FILL if states.prefill_order == "fill" else lv.ORDER_STABLE
    if states.kv_from is not None and states.per_layer:
        for st in states.layers[states.kv_from // w.batch:]:
            ctx.kv_compress(st.k, st.v, st.score, st.kind, st.pos, st.len, mode=lv.KV_THRESHOLD, beta=w.kv_beta,
                            order=order, len_bound=st.N, n_evicted=st.n_evicted, reserve=reserve)
    elif states.kv_from is not None:
        # the threshold rule on the caches of all compressed layers at once (a cache is only read again in decode)
        t = states.tail
        ctx.kv_compress(t(states.k), t(states.v), t(states.score), t(states.kind), t(states.pos), t(states.len),
                        mode=lv.KV_THRESHOLD, beta=w.kv_beta, order=order, len_bound=states.kv_bound,
                        n_evicted=t(states.n_evicted), reserve=reserve)


def run_prefill_budget(ctx, lv, w, states, reserve):
    """Where the workload fixes a per-head budget: every cache of every layer down to it before generation
    starts (one call over the stacked caches; a call no head can exceed the budget in launches nothing)."""
    if w.kv_budget <= 0:
        return
    order = lv.ORDER_FILL if states.prefill_order == "fill" else lv.ORDER_STABLE
    if states.per_layer:
        for st in states:
            ctx.kv_compress(st.k, st.v, st.score, st.kind, st.pos, st.len, mode=lv.KV_BUDGET, budget=w.kv_budget,
                            n_recent=0, order=order, len_bound=st.N, want_evicted=False, reserve=reserve)
    else:
        ctx.kv_compress(states.k, states.v, states.score, states.kind, states.pos, states.len, mode=lv.KV_BUDGET,
                        budget=w.kv_budget, n_recent=0, order=order, len_bound=states.all_bound, want_evicted=False,
                        reserve=reserve)


def run_decode(ctx, lv, w, states, reserve, step_pos=0):
    run_decode_layers(ctx, lv, w, states, reserve, step_pos)
    run_decode_compress(ctx, lv, w, states, reserve)


def decode_evicts_in_attention(w, states):
    """A cache that can be exactly one entry over its budget can be compressed by the attention call itself
    (states.evict == "fused", the default of a state); with "batched" the layers' calls only update the importance
    and ONE lvlm_kv_compress over the stacked caches of all layers evicts at the end of the step -- a layer's cache
    is not read again before the next step."""
    return w.kv_budget > 0 and states.dec_bound == w.kv_budget + 1 and getattr(states, "evict", "fused") == "fused"


def run_decode_layers(ctx, lv, w, states, reserve, step_pos=0):
    fused = decode_evicts_in_attention(w, states)
    for st in states:
        ctx.decode_attn(st.q_dec, st.k_dec, st.v_dec, st.k, st.v, st.score, st.kind, st.pos, st.len,
                        score_decay=0.9, new_pos=w.seq_len + step_pos, len_bound=st.dec_bound, out=st.out_dec,
                        evict_budget=w.kv_budget if fused else 0, evict_recent=1, reserve=reserve)


def run_decode_compress(ctx, lv, w, states, reserve):
    if w.kv_budget > 0 and not decode_evicts_in_attention(w, states) and states.per_layer:
        for st in states:
            ctx.kv_compress(st.k, st.v, st.score, st.kind, st.pos, st.len, mode=lv.KV_BUDGET, budget=w.kv_budget,
                            n_recent=1, order=lv.ORDER_FILL, len_bound=st.dec_bound, want_evicted=False,
                            reserve=reserve)
    elif w.kv_budget > 0 and not decode_evicts_in_attention(w, states):
        # one budget eviction over the caches of all layers (a layer's cache is next read in the next step)
        ctx.kv_compress(states.k, states.v, states.score, states.kind, states.pos, states.len, mode=lv.KV_BUDGET,
                        budget=w.kv_budget, n_recent=1, order=lv.ORDER_FILL, len_bound=states.dec_bound,
                        want_evicted=False, reserve=reserve)


# ----------------------------------------------------------------------------- algorithmic work per kernel
def score_form(ctx, lv, w, N, n_img, batch):
    """The launch form the library takes for `batch` sequences of N keys (lvlm_score_plan: 0 two passes, 1 / 2 one launch,
    3 the shared-tile kernel with the keys in runs, one launch per sweep)."""
    from paper_2509_00419_amd import binding as bd
    d = bd.ScoreDesc(bd.BF16 if w.dtype == "bf16" else bd.F32, batch, N, w.n_text, w.n_sys + n_img, w.n_q_heads,
                     w.n_kv_heads, w.head_dim, w.n_sys, n_img, 1, w.head_dim ** -0.5,
                     w.n_text * w.n_q_heads * w.head_dim, w.n_q_heads * w.head_dim, w.head_dim,
                     N * w.n_kv_heads * w.head_dim, w.n_kv_heads * w.head_dim, w.head_dim, 0, 0)
    return ctx.score_plan(d)


def moved_entries(pos_before, pos_after, len_after, torch):
    """Entries a cache compression moved: slots below the new length whose entry (told by its original position,
    unique per head) is not the one that sat there before.  Arithmetic on copies taken during set-up."""
    L = pos_after.shape[-1]
    live = torch.arange(L, device=pos_after.device)[None, None, :] < len_after[:, :, None]
    return int(((pos_before != pos_after) & live).sum())


def kernel_work(ctx, lv, w, layers, dec_lens, moved, merge="rank", per_layer=False, given_lse=False, fused=False,
                decode_compress=False):
    """Algorithmic bytes / flops of every kernel of one step (summed over its launches), by the profiler's kernel
    names.  HBM kernels: what the method must move, counted once (inputs read once, outputs written once);
    contractions: their multiply-adds.  dec_lens[i]: entries per head of layer i's cache when the decode step
    starts; moved: entries the two compressions at the end of prefill look at and move (counted on one step's state)."""
    e = 2 if w.dtype == "bf16" else 4
    B, Hq, H, d, T = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_text
    work = {}

    def add(name, bound, amount, launches=1):
        a = work.setdefault(name, {"bound": bound, "amount": 0.0, "launches": 0})
        a["amount"] += amount
        a["launches"] += launches

    for first, last in score_groups(layers, per_layer):
        n_img = layers[last]["n_img"]
        N, gb = w.n_sys + n_img + T, (last - first + 1) * B
        form = score_form(ctx, lv, w, N, n_img, gb)
        if form != 0:
            launches = 2 if form == 3 and not given_lse else 1               # form 3: one launch per sweep
            add("score_single", "mfma", 2.0 * gb * T * ((0 if given_lse else N) + n_img) * d * Hq, launches=launches)
            if form == 3 and not given_lse:
                add("score_lse", "hbm", 4.0 * gb * Hq * T)                   # the row normalisers folded in between
        else:
            if not given_lse:
                add("score_pass0", "mfma", 2.0 * gb * T * N * d * Hq)
                add("score_lse", "hbm", 4.0 * gb * Hq * T)                   # the row normalisers it leaves
            add("score_pass1", "mfma", 2.0 * gb * T * n_img * d * Hq)
        add("score_finalize", "hbm", 4.0 * gb * (H + 1) * n_img)             # the scores written
    for i, en in enumerate(layers):
        N = w.n_sys + en["n_img"] + T
        if en["merge_to"] is not None and en["merge_to"] < en["n_img"]:
            r = en["n_img"] - en["merge_to"]
            if merge == "similar":
                rowb, n_img, outside = w.hidden * e + 3 * 4, en["n_img"], N - en["n_img"]
                add("sim_gemm", "mfma", 2.0 * B * r * en["merge_to"] * w.hidden)
                add("sim_rank", "hbm", 8.0 * B * n_img)
                add("sim_rank2", "hbm", 8.0 * B * n_img)
                add("sim_index", "hbm", 8.0 * B * n_img)
                add("sim_order", "hbm", 8.0 * B * n_img)
                add("sim_assign", "hbm", 8.0 * B * n_img)
                add("sim_norm", "hbm", B * n_img * (w.hidden * e + 4.0))            # every image row in, its norm out
                add("sim_merge", "hbm", B * (n_img + en["merge_to"]) * rowb)        # image rows in, dominant rows out
                if outside > 0:
                    add("sim_copy", "hbm", 2.0 * B * outside * rowb)
            else:
                add("merge_rank", "hbm", 8.0 * B * en["n_img"])             # scores in, ranks out
                add("merge_index", "hbm", 8.0 * B * en["n_img"])            # ranks in, index lists out
                add("merge_gather", "hbm", B * (N + N - r) * (w.hidden * e + 3 * 4))
                add("merge_finalize", "hbm", B * w.hidden * e)              # the merged row
        elif en["merge_to"] is not None:                                    # a 100 % stage copies the planes
            add("sim_copy" if merge == "similar" else "merge_gather", "hbm", B * 2 * N * (w.hidden * e + 3 * 4))
        L = float(dec_lens[i].double().mean()) + 1.0
        add("attn_partial", "hbm", 2.0 * B * H * L * d * e)                  # K and V of every retained entry, once
        # the fold: importance read-modify-write of every entry, the queries in, the output rows out
        add("attn_combine_evict" if fused else "attn_combine", "hbm", 8.0 * B * H * L + 2.0 * B * Hq * d * e)
        if decode_compress:                                                  # score and kind of every entry, one entry moved
            add("kv_select", "hbm", B * H * (5.0 * L + 2 * d * e + 9), launches=1.0 / len(layers))
    entry = 2 * d * e + 9                                                   # K row, V row, score, kind, position
    for key in ("threshold", "budget"):
        if moved.get(key + "_scanned", 0) > 0:
            add("kv_select", "hbm", 5.0 * moved[key + "_scanned"])           # score and kind of every entry
        if moved.get(key + "_moved", 0) > 0:                                 # every moved entry read and written
            add("kv_move" if moved.get("order") == "stable" else "kv_fill", "hbm", 2.0 * moved[key + "_moved"] * entry)
    return work


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2509_00419_amd as lv
    from workloads import configs, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    w = configs.ALL[args.workload]
    layers = plan(w, lv)
    ctx = lv.Context(0)
    if args.op == "prefill_attn":
        return main_prefill_attn(args, w, layers, ctx, lv, torch, dev)
    if args.op == "stream":
        return main_stream(args, w, layers, ctx, lv, torch, dev)
    if args.op == "score_load":
        return main_score_load(args, w, layers, ctx, lv, torch, dev)
    t_setup = time.time()
    master = build_master(w, layers, torch, synth, dev, args.row_lse == "given")
    n_first = 3                                   # sets whose first decode step after prefill is timed as well
    n_sets = 1 + args.warmup + args.steps + args.profile_steps
    sets = [StepState(w, layers, master, torch, args.per_layer, args.prefill_order, args.row_lse == "given")
            for _ in range(n_sets)]
    torch.cuda.synchronize()
    print(f"[bench] {w.name}: {len(layers)} layers, {n_sets} state sets, setup {time.time() - t_setup:.1f}s",
          file=sys.stderr, flush=True)

    # dry run on set 0: sizes the workspace, counts the entries the compressions move, gives the cache lengths
    run_prefill_layers(ctx, lv, w, sets[0], reserve=True, merge=args.merge)
    moved = {"order": args.prefill_order}
    p0, l0 = sets[0].pos.clone(), sets[0].len.clone()
    run_prefill_compress(ctx, lv, w, sets[0], reserve=True)
    p1, l1 = sets[0].pos.clone(), sets[0].len.clone()
    kept_fraction = None
    if sets[0].kv_from is not None:
        moved["threshold_scanned"] = int(l0[sets[0].kv_from:].sum())
        moved["threshold_moved"] = moved_entries(p0, p1, l1, torch)
        # share of its image entries each compressed layer keeps under the one threshold (mean over heads)
        kept_fraction = [round(float((st.len.double().mean() - w.n_sys - w.n_text) / st.n_img), 4)
                         for st in sets[0] if st.entry["kv_threshold"]]
    run_prefill_budget(ctx, lv, w, sets[0], reserve=True)
    p2, l2 = sets[0].pos.clone(), sets[0].len.clone()
    if w.kv_budget > 0 and int(l1.max()) > w.kv_budget:
        moved["budget_scanned"] = int(l1.sum())
        moved["budget_moved"] = moved_entries(p1, p2, l2, torch)
    torch.cuda.synchronize()
    lens_after_prefill = [st.len.clone() for st in sets[0]]

    # Steady-state decode: where the budget binds but prefill leaves some heads short of it, the decode phase
    # runs on caches the path itself has filled (set-up, untimed); else on the caches as prefill left them.
    lmin, lmax = int(sets[0].len.min()), int(sets[0].len.max())
    steady = w.kv_budget > 0 and lmax == w.kv_budget and lmin < w.kv_budget
    dec_sets, steady_steps = sets, 0
    if steady:
        t0 = time.time()
        base = SteadyState.from_prefilled(w, torch, synth, ctx, lv, sets[0])
        steady_steps = base.steps_run
        dec_sets = [base] + [base.clone(torch) for _ in range(n_sets - 1)]
        print(f"[bench] steady-state caches: {steady_steps} decode steps run forward in {time.time() - t0:.1f}s",
              file=sys.stderr, flush=True)
        dec_lens = [st.len.clone() for st in base]
    else:
        dec_lens = lens_after_prefill
    for st_ in set(dec_sets) | set(sets):
        st_.evict = args.decode_evict
    run_decode(ctx, lv, w, sets[0], reserve=True)            # (also the first decode step's workspace)
    if steady:
        run_decode(ctx, lv, w, dec_sets[0], reserve=True, step_pos=steady_steps + 1)     # the steady-state shapes' workspace
    torch.cuda.synchronize()
    fused = decode_evicts_in_attention(w, dec_sets[1])
    binds = w.kv_budget > 0 and dec_sets[1].dec_bound == w.kv_budget + 1      # one eviction per head and step

    # capture one (prefill, decode) graph pair per remaining set
    use_graph = not args.no_graph
    has_prefill = any(en["score"] or en["merge_to"] is not None or en["kv_threshold"] for en in layers)
    graphs, first_graphs = [], []
    if use_graph:
        for s in range(1, 1 + args.warmup + args.steps):
            gp, gd = torch.cuda.CUDAGraph() if has_prefill else None, torch.cuda.CUDAGraph()
            if has_prefill:
                with torch.cuda.graph(gp):
                    run_prefill(ctx, lv, w, sets[s], reserve=False, merge=args.merge)
            with torch.cuda.graph(gd):
                run_decode(ctx, lv, w, dec_sets[s], reserve=False, step_pos=steady_steps + 1)
            graphs.append((gp, gd))
        if steady:
            for s in range(1, 1 + min(n_first, args.warmup + args.steps)):
                gf = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gf):
                    run_decode(ctx, lv, w, sets[s], reserve=False)
                first_graphs.append(gf)
        torch.cuda.synchronize()

    def step(i):
        if use_graph:
            if has_prefill:
                graphs[i][0].replay()
            ev_mid[i].record()
            graphs[i][1].replay()
        else:
            run_prefill(ctx, lv, w, sets[1 + i], reserve=False, merge=args.merge)
            ev_mid[i].record()
            run_decode(ctx, lv, w, dec_sets[1 + i], reserve=False, step_pos=steady_steps + 1)

    n_run = args.warmup + args.steps
    ev_mid = [torch.cuda.Event(enable_timing=True) for _ in range(n_run)]
    ev_beg = [torch.cuda.Event(enable_timing=True) for _ in range(n_run + 1)]
    for i in range(args.warmup):
        ev_beg[i].record()
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, n_run):
        ev_beg[i].record()
        step(i)
    ev_beg[n_run].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    prefill_ms = sum(ev_beg[i].elapsed_time(ev_mid[i]) for i in range(args.warmup, n_run)) / args.steps
    decode_ms = sum(ev_mid[i].elapsed_time(ev_beg[i + 1]) for i in range(args.warmup, n_run)) / args.steps

    # the first decode step after prefill (caches as prefill left them), outside the timed region
    first_ms = None
    if first_graphs:
        ta, tb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        tot = 0.0
        for gf in first_graphs:
            torch.cuda.synchronize()
            ta.record()
            gf.replay()
            tb.record()
            torch.cuda.synchronize()
            tot += ta.elapsed_time(tb)
        first_ms = tot / len(first_graphs)

    # per-kernel durations: eager steps in which every launch carries HIP events bound to the kernel itself, on the
    # launch stream (first wave to last wave, as a kernel trace reports it)
    prof = {}
    if args.profile_steps > 0:
        ctx.profile(True)
        agg = {}
        for s in range(1 + n_run, n_sets):
            run_prefill(ctx, lv, w, sets[s], reserve=False, merge=args.merge)
            for name, (calls, tot, mn, mx) in ctx.profile_read().items():
                a = agg.setdefault(name, [0, 0.0])
                a[0] += calls
                a[1] += tot
            run_decode(ctx, lv, w, dec_sets[s], reserve=False, step_pos=steady_steps + 1)
            for name, (calls, tot, mn, mx) in ctx.profile_read().items():
                a = agg.setdefault(name, [0, 0.0])
                a[0] += calls
                a[1] += tot
        ctx.profile(False)
        prof = {k: {"launches_per_step": v[0] / args.profile_steps, "us_per_step": v[1] * 1e3 / args.profile_steps,
                    "avg_us": v[1] * 1e3 / max(v[0], 1)} for k, v in agg.items()}

    if args.copy_calibration:
        # a copy large enough that the lines still dirty in the L2s when it ends (tens of MB) do not matter
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)           # one device copy: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()

    mfma_peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS
    work = kernel_work(ctx, lv, w, layers, dec_lens, moved, args.merge, args.per_layer, args.row_lse == "given", fused,
                       decode_compress=binds and not fused)
    kernels = {}
    for name, p in sorted(prof.items(), key=lambda kv: -kv[1]["us_per_step"]):
        row = {"avg_us": round(p["avg_us"], 2), "launches_per_step": p["launches_per_step"],
               "us_per_step": round(p["us_per_step"], 1)}
        if name in work and p["us_per_step"] > 0:
            amt = work[name]["amount"]
            if name.startswith("score_") and name != "score_finalize" and \
                    abs(p["launches_per_step"] - work[name]["launches"]) > 1e-9:
                raise SystemExit(f"bench: {name} ran {p['launches_per_step']} times per step, the work model "
                                 f"expects {work[name]['launches']}")
            if work[name]["bound"] == "hbm":
                row.update(bound="hbm", achieved_GBs=round(amt / p["us_per_step"] / 1e3, 1),
                           frac=round(amt / p["us_per_step"] / 1e3 / HBM_PEAK_GBS, 4))
            else:
                row.update(bound="mfma", achieved_TFLOPs=round(amt / p["us_per_step"] / 1e6, 1),
                           frac=round(amt / p["us_per_step"] / 1e6 / mfma_peak, 4))
        kernels[name] = row
    # The dominant kernel: the one with the most time per step among ALL kernels of the path.  `traffic` (HBM
    # bytes by the rocprofv3 counters) is not measured inside this run: it is null here and stands, per kernel
    # and shape, in the profiler summaries kept beside the sources.
    roofline = None
    for name, row in kernels.items():
        if "bound" not in row:
            raise SystemExit(f"bench: kernel {name} has no work model")
        amt, per_launch = work[name]["amount"], max(row["launches_per_step"], 1)
        if row["bound"] == "hbm":
            roofline = {"kernel": name, "bound": "hbm", "achieved": row["achieved_GBs"], "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": row["frac"], "traffic": None,
                        "algorithmic_bytes_per_launch": amt / per_launch, "avg_launch_us": row["avg_us"]}
        else:
            roofline = {"kernel": name, "bound": "mfma", "achieved": row["achieved_TFLOPs"],
                        "peak": mfma_peak, "unit": "TFLOP/s", "frac": row["frac"], "traffic": None,
                        "algorithmic_flops_per_launch": amt / per_launch, "avg_launch_us": row["avg_us"]}
        break
    # the decode layer-step as a whole (both attention kernels) against the bytes of its K and V rows
    decode_layer = None
    if "attn_partial" in kernels:
        us = sum(kernels[k]["us_per_step"] for k in ("attn_partial", "attn_combine", "attn_combine_evict") if k in kernels)
        amt = sum(work[k]["amount"] for k in ("attn_partial", "attn_combine", "attn_combine_evict") if k in work)
        decode_layer = {"us_per_layer": round(us / len(layers), 2), "algorithmic_bytes_per_layer": amt / len(layers),
                        "achieved_GBs": round(amt / us / 1e3, 1), "frac": round(amt / us / 1e3 / HBM_PEAK_GBS, 4)}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, layers, master, torch, lv, args.merge, dec_sets[0] if steady else None, steady_steps)

    out = {
        "metric": "prefill merge tokens/s + compacted-KV decode steps/s; % HBM roofline",
        "value": round(w.batch * w.n_img / (ms_per_step * 1e-3), 1),
        "unit": "image tokens/s (whole step: prefill token reduction + one steady-state decode step over all layers)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "layers": w.layers, "seq": [w.n_sys, w.n_img, w.n_text],
                   "image_tokens_per_layer": [en["n_img"] for en in layers if en["merge_to"] is not None] +
                                             [layers[-1]["n_img"]],
                   "kv_beta": w.kv_beta, "kv_budget": w.kv_budget, "merge": args.merge, "graphs": use_graph,
                   "calls": "per layer" if args.per_layer else "batched over layers",
                   "prefill_order": args.prefill_order, "row_lse": args.row_lse,
                   "decode_state": (f"steady state: every head at its budget of {w.kv_budget} entries (caches filled by "
                                    f"{steady_steps} decode steps of the path during set-up)") if steady else
                                   ("steady state: every head at its budget as prefill leaves it" if fused else
                                    "caches as prefill leaves them (the budget does not bind)"),
                   "eviction": "inside lvlm_decode_attn" if fused else
                               ("one lvlm_kv_compress over all layers' caches at the end of the step" if binds else "none needed"),
                   "image_entries_kept_by_threshold_per_layer": kept_fraction},
        "prefill_ms": round(prefill_ms, 4), "decode_step_ms": round(decode_ms, 4),
        "prefill_image_tokens_per_s": round(w.batch * w.n_img / (prefill_ms * 1e-3), 1) if prefill_ms > 0 else None,
        "decode_steps_per_s": round(1e3 / decode_ms, 1),
        "first_decode_step_after_prefill_ms": None if first_ms is None else round(first_ms, 4),
        "decode_layer_step": decode_layer,
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels,
    }
    print(json.dumps(out))


# ----------------------------------------------------------------------------- the score call against its load
def main_score_load(args, w, layers, ctx, lv, torch, dev):
    """--op score_load: lvlm_score_tokens alone, random queries and keys of the workload's head shape, at every
    token count the pyramid leaves behind its merge layers, for 4 to 32 sequences per call (the bench's own calls
    stack the layers of a run on that axis).  Reports the main kernel's duration (events bound to the kernels),
    the workgroups the one-launch form starts (a workgroup = four 32-row query chunks of one KV head) and the
    fraction of the bf16 MFMA peak: the time is a staircase in the workgroups per compute unit."""
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else MFMA_F32_PEAK_TFLOPS
    Hq, Hkv, d, T = w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_text
    n_chunks = (Hq // Hkv * T + 31) // 32
    shapes = sorted({en["merge_to"] for en in layers if en["merge_to"] is not None}, reverse=True)
    shapes = shapes or [w.n_img]                       # a workload that merges nothing: its full image span
    rows = []
    for n_img in shapes:
        N = w.n_sys + n_img + T
        for B in (4, 8, 10, 12, 14, 16, 20, 24, 32):
            torch.manual_seed(B)
            q = torch.randn(B, T, Hq, d, device=dev, dtype=dt)
            k = torch.randn(B, N, Hkv, d, device=dev, dtype=dt)
            sh = torch.empty(B, Hkv, n_img, dtype=torch.float32, device=dev)
            sm = torch.empty(B, n_img, dtype=torch.float32, device=dev)
            kw = dict(q_pos0=w.n_sys + n_img, img_begin=w.n_sys, n_img=n_img, score_head=sh, score_mean=sm)
            form = ctx.score_plan(ctx.score_desc(q, k, q_pos0=kw["q_pos0"], img_begin=kw["img_begin"], n_img=n_img))
            ctx.score_tokens(q, k, **kw)
            torch.cuda.synchronize()
            ctx.profile(True)
            for _ in range(args.steps):
                ctx.score_tokens(q, k, **kw)
            torch.cuda.synchronize()
            got = ctx.profile_read()
            ctx.profile(False)
            us = sum(v[1] for kk, v in got.items() if kk in ("score_single", "score_pass0", "score_pass1")) * 1e3 / args.steps
            flops = 2.0 * B * Hq * T * d * (N + n_img)
            wgs = B * Hkv * ((n_chunks + 3) // 4)
            rows.append({"n_img": n_img, "keys": N, "sequences": B, "form": ["two passes", "one launch, a chunk per workgroup",
                                                                           "one launch, shared tiles",
                                                                           "shared tiles, keys in runs"][form],
                         "workgroups": wgs if form >= 2 else None,
                         "workgroups_per_cu": round(wgs / 256, 2) if form >= 2 else None, "us": round(us, 1),
                         "TFLOPs": round(flops / us / 1e6, 1), "frac_of_peak": round(flops / us / 1e6 / peak, 4)})
            del q, k, sh, sm
    best = max(rows, key=lambda r: r["TFLOPs"])
    print(json.dumps({
        "metric": "lvlm_score_tokens alone against the sequences per call", "value": best["TFLOPs"],
        "unit": "TFLOP/s (best sequence count)", "n_gpus": 1, "steps": args.steps, "warmup": 1, "higher_is_better": True,
        "dtype": w.dtype, "data": "synthetic (random queries and keys)",
        "config": {"workload": w.name, "Hq": Hq, "Hkv": Hkv, "head_dim": d, "instruction_rows": T,
                   "query_chunks_per_kv_head": n_chunks},
        "rows": rows}))


# ----------------------------------------------------------------------------- what a launch can stream
def main_stream(args, w, layers, ctx, lv, torch, dev):
    """--op stream: the read-only probe over one buffer per layer, each as large as the K and V rows one decode
    launch of the workload reads (B x Hkv x (budget or sequence) x 2 rows), launched back to back over the layers
    like the decode step, for a range of workgroup counts; then ONE workgroup over 1 MiB (what one compute unit
    streams).  Durations from events bound to the kernels."""
    e = 2 if w.dtype == "bf16" else 4
    entries = (w.kv_budget + 1) if w.kv_budget > 0 else w.seq_len + 1
    nbytes = w.batch * w.n_kv_heads * entries * 2 * w.head_dim * e // 16 * 16
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(len(layers))]
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    rows = []
    ctx.profile(True)
    for n_wg in (64, 128, 256, 512, 1024, 2048, 4096):
        for rep in range(1 + args.steps):
            for b in bufs:
                ctx.stream_probe(b, n_wg, sink)
            torch.cuda.synchronize()
            got = ctx.profile_read()["stream_probe"]
            if rep == 0:
                continue                                   # warm-up round
            rows.append((n_wg, got[0], got[1] * 1e3 / got[0]))
    one = torch.empty(1 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    for rep in range(1 + args.steps):
        for _ in range(16):
            ctx.stream_probe(one, 1, sink)
        torch.cuda.synchronize()
        got = ctx.profile_read()["stream_probe"]
        single_us = got[1] * 1e3 / got[0]
    ctx.profile(False)
    # the yardstick of the gather: a plain device copy (torch's) that moves as many bytes, read + written, as each
    # merge stage of the workload does (hidden and position planes: every source row in, every surviving row out)
    copies = []
    for en in layers:
        if en["merge_to"] is None or en["merge_to"] >= en["n_img"]:
            continue
        Nq = w.n_sys + en["n_img"] + w.n_text
        moved = w.batch * (Nq + Nq - (en["n_img"] - en["merge_to"])) * (w.hidden * e + 12)
        half = moved // 2 // 16 * 16
        # (a different pair of buffers per copy, a GiB of them in all: a repeated copy of one pair would be served
        # in part by the last-level cache, which the gather's rows, written by other kernels long before, are not)
        n_pairs = max(2, -(-(1 << 30) // (2 * half)))
        pairs = [tuple(torch.empty(half, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(2))
                 for _ in range(n_pairs)]
        reps = n_pairs * (1 + args.steps)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i_, (a_, b_) in enumerate(evs):
            src_, dst_ = pairs[i_ % n_pairs]
            a_.record(); dst_.copy_(src_); b_.record()
        torch.cuda.synchronize()
        timed = evs[n_pairs:]
        us = sum(a_.elapsed_time(b_) for a_, b_ in timed) * 1e3 / len(timed)
        copies.append({"stage": f"{en['n_img']} -> {en['merge_to']}", "bytes_read_plus_written": 2 * half, "us": round(us, 2),
                       "GBs": round(2 * half / us / 1e3, 1), "frac_of_peak": round(2 * half / us / 1e3 / HBM_PEAK_GBS, 4)})
        del pairs, src_, dst_
    table = {}
    for n_wg, calls, us in rows:
        table.setdefault(n_wg, []).append(us)
    by_wg = {str(k): {"us_per_launch": round(sum(v) / len(v), 2), "GBs": round(nbytes / (sum(v) / len(v)) / 1e3, 1),
                      "frac_of_peak": round(nbytes / (sum(v) / len(v)) / 1e3 / HBM_PEAK_GBS, 4)} for k, v in table.items()}
    best = max(by_wg.values(), key=lambda r: r["GBs"])
    print(json.dumps({
        "metric": "read-only streaming probe (lvlm_stream_probe)", "value": best["GBs"], "unit": "GB/s (best workgroup count)",
        "n_gpus": 1, "steps": args.steps, "warmup": 1, "higher_is_better": True, "dtype": "u8", "data": "synthetic",
        "config": {"workload": w.name, "bytes_per_launch": nbytes, "launches": len(layers),
                   "what": "one decode layer's K and V rows per launch, a different buffer per launch"},
        "by_workgroups": by_wg,
        "one_workgroup_1MiB": {"us": round(single_us, 2), "GBs": round((1 << 20) / single_us / 1e3, 1)},
        "device_copy_of_merge_stage_bytes": copies,
        "roofline": {"bound": "hbm", "achieved": best["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": best["frac_of_peak"], "traffic": None}}))


# ----------------------------------------------------------------------------- the layers' own attention
def main_prefill_attn(args, w, layers, ctx, lv, torch, dev):
    """--op prefill_attn: one step = lvlm_prefill_attn for every layer of the stack, layer l on the
    n_sys + n_img(l) + n_text tokens the pyramid has left at its input, with the scores of the instruction rows
    as by-product at the layers the path scores.  The same stack without merging (every layer at the full
    sequence) is timed beside it: the ratio is the attention share of the paper's prefill saving.
    q, k, v are views of one fused projection output [B, N, Hq + 2 Hkv, d] (four buffers taken in turn)."""
    Hq, Hkv, d, B, T = w.n_q_heads, w.n_kv_heads, w.head_dim, w.batch, w.n_text
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    Nmax = w.seq_len
    g = torch.Generator(device=dev).manual_seed(w.seed)
    fused = [torch.randn(B, Nmax, Hq + 2 * Hkv, d, generator=g, device=dev).to(dt) for _ in range(4)]
    out = torch.empty(B, Nmax, Hq, d, dtype=dt, device=dev)
    lse = torch.empty(B * Hq * Nmax, dtype=torch.float32, device=dev)
    sizes = sorted({en["n_img"] for en in layers} | {w.n_img})
    sh = {n: torch.empty(B, Hkv, n, dtype=torch.float32, device=dev) for n in sizes}
    sm = {n: torch.empty(B, n, dtype=torch.float32, device=dev) for n in sizes}

    def run(merged, reserve=False):
        for li, en in enumerate(layers):
            n_img = en["n_img"] if merged else w.n_img
            N = w.n_sys + n_img + T
            f = fused[li % 4][:, :N]
            scored = en["score"] and n_img > 0
            ctx.prefill_attn(f[:, :, :Hq], f[:, :, Hq:Hq + Hkv], f[:, :, Hq + Hkv:], n_text=T if scored else 0,
                             img_begin=w.n_sys, n_img=n_img, out=out[:, :N], row_lse=lse[:B * Hq * N].view(B, Hq, N),
                             score_head=sh[n_img] if scored else None, score_mean=sm[n_img] if scored else None,
                             reserve=reserve)

    def timed(merged, steps, warmup):
        for _ in range(warmup):
            run(merged)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run(merged)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    run(False, reserve=True)
    run(True, reserve=True)
    torch.cuda.synchronize()
    ms_per_step = timed(True, args.steps, args.warmup)
    ms_unmerged = timed(False, max(1, args.steps // 4), 1)

    # per-kernel durations: HIP events on the launch stream around every launch
    prof = {}
    if args.profile_steps > 0:
        ctx.profile(True)
        for _ in range(args.profile_steps):
            run(True)
        torch.cuda.synchronize()
        prof = {k: {"launches_per_step": v[0] / args.profile_steps, "us_per_step": v[1] * 1e3 / args.profile_steps,
                    "avg_us": v[1] * 1e3 / max(v[0], 1)} for k, v in ctx.profile_read().items()}
        ctx.profile(False)
    counts = [w.n_sys + en["n_img"] + T for en in layers]
    flops = sum(4.0 * B * Hq * d * n * (n + 1) / 2 for n in counts)        # causal: row i multiplies i + 1 keys, twice
    kernels = {k: {"avg_us": round(v["avg_us"], 2), "launches_per_step": v["launches_per_step"],
                   "us_per_step": round(v["us_per_step"], 1)} for k, v in sorted(prof.items(), key=lambda kv: -kv[1]["us_per_step"])}
    roofline = None
    if "prefill_attn" in prof:
        p = prof["prefill_attn"]
        tf = flops / p["us_per_step"] / 1e6
        peak = MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else 157.3
        kernels["prefill_attn"].update(bound="mfma", achieved_TFLOPs=round(tf, 1),
                                       frac=round(tf / peak, 4))
        roofline = {"kernel": "prefill_attn", "bound": "mfma", "achieved": round(tf, 1),
                    "peak": peak, "unit": "TFLOP/s", "frac": round(tf / peak, 4), "traffic": None,
                    "algorithmic_flops_per_launch": flops / len(layers), "avg_launch_us": round(p["avg_us"], 2)}
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import lvlm_oracle as O
        # the oracle on one sequence of one layer of the stack (the longest of at most 6000 tokens) and as many KV
        # groups as keep the sample near ten seconds, scaled by causal flops to the whole stack
        fit = [n for n in counts if n <= 6000]
        N = max(fit) if fit else min(counts)
        li = counts.index(N)
        G = Hq // Hkv
        ng = max(1, min(Hkv, int(2e8 / (float(N) * N * G))))
        f = fused[li % 4][:1, :N].double().cpu().numpy()
        t0 = time.perf_counter()
        O.prefill_attn(f[:, :, :ng * G], f[:, :, Hq:Hq + ng], f[:, :, Hq + Hkv:Hq + Hkv + ng], dtype=w.dtype)
        t = time.perf_counter() - t0
        sample_flops = 4.0 * ng * G * d * N * (N + 1) / 2
        cpu = {"value": round(B * w.n_img / (t * flops / sample_flops), 2), "unit": "image tokens/s", "cores": os.cpu_count(),
               "kind": "oracle", "sample": f"oracle.prefill_attn on one sequence of layer {li} ({N} tokens), {ng} KV "
               f"group(s) = {ng * G} query heads: {t:.2f} s, scaled by causal flops to the whole stack"}
    print(json.dumps({
        "metric": "prefill attention with scores as by-product, over the layer stack",
        "value": round(B * w.n_img / (ms_per_step * 1e-3), 1), "unit": "image tokens/s (attention of all layers)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "op": "prefill_attn", "batch": B, "layers": w.layers, "seq": [w.n_sys, w.n_img, T],
                   "tokens_per_layer": counts},
        "ms_per_step_without_merging": round(ms_unmerged, 4), "attention_speedup_from_merging": round(ms_unmerged / ms_per_step, 3),
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels}))


# ----------------------------------------------------------------------------- oracle leg
def cpu_baseline(w, layers, master, torch, lv, merge="rank", steady=None, steady_steps=0):
    """The oracle, as it stands, on one full step of the same inputs (host cores): prefill of every layer, the
    compressions, and one decode step (on the steady-state caches where the bench decodes on those)."""
    import numpy as np

    from oracle import lvlm_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1

    def f64(t):
        return t.detach().double().cpu().numpy()

    def host_of(m):
        return {k: (f64(v) if v.dtype in (torch.bfloat16, torch.float32) else v.cpu().numpy()) for k, v in m.items()}

    # a bounded sample: every layer of the small stacks, every stride-th layer of the large ones (each run of
    # layers with one token count keeps several), scaled by the stride
    stride = -(-len(layers) // 12) if w.n_img * w.layers * w.batch > 200_000 else 1
    sec, n_done = 0.0, 0
    for li, (en, m) in enumerate(zip(layers, master)):
        if li % stride:
            continue
        n_done += 1
        m = host_of(m)                           # one layer on the host at a time (config 5: 0.5 GB in fp64)
        dec = None
        if steady is not None:
            L = steady[li]
            dec = [f64(L.k), f64(L.v), L.score.cpu().numpy(), L.kind.cpu().numpy(), L.pos.cpu().numpy(),
                   L.len.cpu().numpy(), f64(L.q_dec), f64(L.k_dec), f64(L.v_dec)]
        t0 = time.perf_counter()
        N = w.n_sys + en["n_img"] + w.n_text
        img0 = w.n_sys
        if en["score"]:
            k = np.transpose(m["k"][:, :, :N], (0, 2, 1, 3))
            sh, sm = O.score_tokens(m["q"], k, q_pos0=img0 + en["n_img"], img_begin=img0, n_img=en["n_img"])
            m["score"][:, :, img0:img0 + en["n_img"]] = sh
        if en["merge_to"] is not None and merge == "similar":
            O.merge_similar([m["hidden"], m["pos_ids"]], sm, img_begin=img0, n_img=en["n_img"],
                            n_keep=en["merge_to"], rules=[O.RULE_WEIGHTED, O.RULE_TOP], dtypes=[w.dtype, "f32"])
        elif en["merge_to"] is not None:
            O.merge_compact([m["hidden"], m["pos_ids"]], sm, img_begin=img0, n_img=en["n_img"],
                            n_keep=en["merge_to"], rules=[O.RULE_WEIGHTED, O.RULE_TOP], dtypes=[w.dtype, "f32"])
        state = [m["k"], m["v"], m["score"].astype(np.float32), m["kind"], m["pos"], m["len"]]
        if en["kv_threshold"]:
            state = list(O.kv_compress(*state, mode="threshold", beta=w.kv_beta, order=O.ORDER_FILL)[:6])
        if w.kv_budget > 0:
            state = list(O.kv_compress(*state, mode="budget", budget=w.kv_budget, n_recent=0, order=O.ORDER_FILL)[:6])
        if dec is not None:
            state, (qd, kd, vd) = dec[:6], dec[6:]
        else:
            qd, kd, vd = m["q_dec"], m["k_dec"], m["v_dec"]
        res = O.decode_attn(qd, kd, vd, *state, score_decay=0.9, new_pos=w.seq_len + steady_steps + 1, out_dtype=w.dtype)
        if w.kv_budget > 0:
            O.kv_compress(*res[1:], mode="budget", budget=w.kv_budget, n_recent=1, order=O.ORDER_FILL)
        sec += time.perf_counter() - t0
    est = sec * len(layers) / n_done
    what = f"all {w.layers} layers" if stride == 1 else \
        f"every {stride}th layer ({n_done} of {w.layers}: {sec:.2f} s), scaled by {len(layers)}/{n_done}"
    return {"value": round(w.batch * w.n_img / est, 1), "unit": "image tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"one step of {w.name} on the same inputs (prefill reduction, cache compressions, one decode "
                      f"step), {what}: {est:.2f} s per step"}


if __name__ == "__main__":
    main()
