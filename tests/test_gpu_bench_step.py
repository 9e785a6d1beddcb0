"""The step that bench.py times, at full size and in its own launch configuration, against the oracle.

bench.py scores runs of layers in one call (layers stacked on the batch axis, keys read through strided
views of the stacked head-major caches), compresses the caches of all layers in one call and decodes layer
by layer.  These tests drive bench.py's own functions on one step's state and check every phase against
the oracle applied to the state the GPU had just before that phase (so one flipped near-tie cannot
cascade): scores within 1e-5, index lists and cache moves exact, values within the dtype's tolerance.
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


def f64(t):
    return t.detach().double().cpu().numpy()


def rel_err(got, ref):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def snapshot(k, v, score, kind, pos, length):
    return [f64(k), f64(v), score.cpu().numpy().copy(), kind.cpu().numpy().copy(), pos.cpu().numpy().copy(),
            length.cpu().numpy().copy()]


def same_entries(now, ref, exact_score=True, tol=1e-5):
    """Caches `now` and `ref` ([k, v, score, kind, pos, len]) hold the same retained entries, slot by slot."""
    assert np.array_equal(now[5], ref[5])
    nb, nh = now[5].shape
    for b in range(nb):
        for h in range(nh):
            n = int(now[5][b, h])
            for i in (0, 1, 3, 4):
                assert np.array_equal(now[i][b, h, :n], ref[i][b, h, :n]), (b, h, i)
            if exact_score:
                assert np.array_equal(now[2][b, h, :n], ref[2][b, h, :n]), (b, h)
            elif n:
                assert rel_err(now[2][b, h, :n], ref[2][b, h, :n]) < tol, (b, h)


def build(w, given_lse=False, prefill_order="fill"):
    layers = bench.plan(w, lv)
    master = bench.build_master(w, layers, torch, synth, DEV, given_lse)
    return layers, master, bench.StepState(w, layers, master, torch, prefill_order=prefill_order, given_lse=given_lse)


def layer_slices(st, i, B):
    sl = slice(i * B, (i + 1) * B)
    return st.k[sl], st.v[sl], st.score[sl], st.kind[sl], st.pos[sl], st.len[sl]


@pytest.mark.parametrize("name,every_layer,given_lse", [("cfg2", True, False), ("cfg3", False, False),
                                                        ("cfg5", False, False), ("cfg2", True, True),
                                                        ("cfg6", False, False)])
def test_prefill_and_decode_step_in_bench_configuration(name, every_layer, given_lse):
    """Config 2: every layer of the step.  Configs 3, 5 and 6 (B = 8; 16512 tokens; the 38B shape with a
    video-like input, G = 5): the first and last layer of every scoring run plus one uncompressed layer -- the
    oracle needs seconds per layer there.  given_lse: the
    bench's --row-lse given mode (row normalisers from plain torch, as an attention kernel would leave them)."""
    w = configs.ALL[name]
    ctx = lv.Context(0)
    layers, master, st = build(w, given_lse)
    B, img0, tol = w.batch, w.n_sys, 2e-2
    if every_layer:
        assert st.groups == [(5, 9), (10, 13), (14, 27)]      # the 100 % stage at layer 5 ends no run
        sample = list(range(len(layers)))
    else:
        sample = sorted({0} | {i for g in st.groups for i in g})

    # ---- prefill, scoring and merging
    bench.run_prefill_layers(ctx, lv, w, st, reserve=True)
    torch.cuda.synchronize()
    for first, last in st.groups:
        for i in range(first, last + 1):
            if i not in sample:
                continue
            L, m = st[i], master[i]
            k = m["k"][:, :, :L.N].permute(0, 2, 1, 3)
            osh, osm = O.score_tokens(f64(m["q"]), f64(k), q_pos0=img0 + L.n_img, img_begin=img0, n_img=L.n_img)
            assert rel_err(L.score[:, :, img0:img0 + L.n_img].cpu(), osh) < 1e-5, i
            rows = st.group_mean[last][(i - first) * B:(i - first + 1) * B]
            assert rel_err(rows.cpu(), osm) < 1e-5, i
    n_merges = 0
    for i, L in enumerate(st):
        e = L.entry
        if e["merge_to"] is None:
            continue
        n_merges += 1
        m = master[i]
        oouts, okeep, omerged = O.merge_compact([f64(m["hidden"]), m["pos_ids"].cpu().numpy()],
                                                np.zeros((B, L.n_img), np.float32) if L.score_mean is None
                                                else L.score_mean.cpu().numpy(), img_begin=img0, n_img=L.n_img,
                                                n_keep=e["merge_to"], rules=[lv.RULE_WEIGHTED, lv.RULE_TOP],
                                                dtypes=[w.dtype, "f32"])
        if e["merge_to"] < L.n_img:
            assert np.array_equal(L.keep_idx.cpu().numpy(), okeep), i
            assert np.array_equal(L.merged_idx.cpu().numpy(), omerged), i
        assert rel_err(f64(L.hidden_out), oouts[0]) < tol, i
        assert np.array_equal(L.pos_out.cpu().numpy(), oouts[1]), i
    assert n_merges == 3

    # ---- prefill, threshold compression of the caches of all compressed layers in one call, on the GPU's
    # score bits (holes filled from the tail: the order the bench runs by default)
    compressed = [i for i in sample if layers[i]["kv_threshold"]]
    before = {i: snapshot(*layer_slices(st, i, B)) for i in compressed}
    bench.run_prefill_compress(ctx, lv, w, st, reserve=True)
    torch.cuda.synchronize()
    shrunk = False
    for i in compressed:
        ref = O.kv_compress(*before[i], mode="threshold", beta=w.kv_beta, order=O.ORDER_FILL)
        now = snapshot(*layer_slices(st, i, B))
        same_entries(now, ref[:6])
        assert np.array_equal(st.n_evicted[i * B:(i + 1) * B].cpu().numpy(), ref[6])
        shrunk = shrunk or bool((now[5] < before[i][5]).any())
    assert shrunk

    # ---- prefill, last call: every cache of every layer down to the budget before generation starts
    before = {i: snapshot(*layer_slices(st, i, B)) for i in sample}
    bench.run_prefill_budget(ctx, lv, w, st, reserve=True)
    torch.cuda.synchronize()
    for i in sample:
        now = snapshot(*layer_slices(st, i, B))
        if w.kv_budget > 0:
            ref = O.kv_compress(*before[i], mode="budget", budget=w.kv_budget, n_recent=0, order=O.ORDER_FILL)
            same_entries(now, ref[:6])
            assert int(now[5].max()) <= w.kv_budget
        else:
            same_entries(now, before[i])
    if name in ("cfg5", "cfg6"):
        # shallow layers full, deep ones short: what the pyramid and the threshold rule left of 492 + text entries
        assert int(st.len.max()) == w.kv_budget and 128 < int(st.len.min()) <= 492 + w.n_text

    # ---- the first decode step after prefill: attention layer by layer with the eviction of one entry inside the
    # call where a head is over its budget afterwards (else one budget eviction over all caches, which finds
    # nothing to do where the budget does not bind).  The same calls without eviction on copies of the sampled
    # layers give the GPU's updated score bits for the oracle to evict on.
    fused = bench.decode_evicts_in_attention(w, st)
    assert fused == (name in ("cfg5", "cfg6"))
    before, mid = {}, {}
    for i in sample:
        L, m = st[i], master[i]
        before[i] = snapshot(*layer_slices(st, i, B))
        cp = [t.clone() for t in layer_slices(st, i, B)]
        plain = ctx.decode_attn(L.q_dec, L.k_dec, L.v_dec, *cp, score_decay=0.9, new_pos=w.seq_len, len_bound=L.dec_bound)
        torch.cuda.synchronize()
        mid[i] = (snapshot(*cp), plain)
        ref = O.decode_attn(f64(m["q_dec"]), f64(m["k_dec"]), f64(m["v_dec"]), *before[i], score_decay=0.9,
                            new_pos=w.seq_len, out_dtype="bf16")
        assert rel_err(f64(plain), ref[0]) < tol, i
        same_entries(mid[i][0], list(ref[1:]), exact_score=False)
    bench.run_decode(ctx, lv, w, st, reserve=True)
    torch.cuda.synchronize()
    for i in sample:
        assert torch.equal(st[i].out_dec, mid[i][1]), i
        now = snapshot(*layer_slices(st, i, B))
        if w.kv_budget > 0:
            ref = O.kv_compress(*mid[i][0], mode="budget", budget=w.kv_budget, n_recent=1, order=O.ORDER_FILL)
            same_entries(now, ref[:6])
            assert int(now[5].max()) <= w.kv_budget
        else:
            same_entries(now, mid[i][0])


def test_steady_state_caches_of_config5_and_one_step_on_them():
    """The decode phase the bench times at config 5: caches that the path itself filled to the budget (budget minus the
    shortest head's length decode steps with eviction, run forward from the prefilled state on every layer), then one more step, checked on the
    first and the last layer against the oracle applied to the GPU state just before it."""
    w = configs.CFG5
    ctx = lv.Context(0)
    layers, master, st = build(w)
    bench.run_prefill(ctx, lv, w, st, reserve=True)
    torch.cuda.synchronize()
    shortest = int(st.len.min())
    assert 128 < shortest <= 492 + w.n_text
    steady = bench.SteadyState.from_prefilled(w, torch, synth, ctx, lv, st)
    assert steady.steps_run == w.kv_budget - shortest
    assert int(steady.len.min()) == w.kv_budget == int(steady.len.max())
    assert bench.decode_evicts_in_attention(w, steady)
    B = w.batch
    # generated entries have displaced image entries in the deep layers, protected text entries are all still there
    for i in (0, len(layers) - 1):
        kinds = steady[i].kind[:, :, :w.kv_budget]
        assert int((kinds == lv.KIND_PROTECTED).sum()) == B * w.n_kv_heads * w.n_text
    assert int((steady[len(layers) - 1].kind[:, :, :w.kv_budget] == lv.KIND_GENERATED).sum()) > 0
    sample = (0, len(layers) - 1)
    before, mid = {}, {}
    for i in sample:
        L = steady[i]
        state = (L.k, L.v, L.score, L.kind, L.pos, L.len)
        before[i] = snapshot(*state)
        cp = [t.clone() for t in state]
        plain = ctx.decode_attn(L.q_dec, L.k_dec, L.v_dec, *cp, score_decay=0.9, new_pos=w.seq_len + steady.steps_run + 1,
                                len_bound=w.kv_budget + 1)
        torch.cuda.synchronize()
        mid[i] = (snapshot(*cp), plain)
        ref = O.decode_attn(f64(L.q_dec), f64(L.k_dec), f64(L.v_dec), *before[i], score_decay=0.9,
                            new_pos=w.seq_len + steady.steps_run + 1, out_dtype="bf16")
        assert rel_err(f64(plain), ref[0]) < 2e-2, i
        same_entries(mid[i][0], list(ref[1:]), exact_score=False)
    bench.run_decode(ctx, lv, w, steady, reserve=True, step_pos=steady.steps_run + 1)
    torch.cuda.synchronize()
    for i in sample:
        L = steady[i]
        assert torch.equal(L.out_dec, mid[i][1])
        ref = O.kv_compress(*mid[i][0], mode="budget", budget=w.kv_budget, n_recent=1, order=O.ORDER_FILL)
        same_entries(snapshot(L.k, L.v, L.score, L.kind, L.pos, L.len), ref[:6])
    assert int(steady.len.min()) == w.kv_budget == int(steady.len.max())
    # the form the bench times by default -- the layers' calls update the importance, ONE lvlm_kv_compress over the
    # stacked caches of all layers evicts at the end of the step -- must leave exactly what the fused form leaves
    other = steady.clone(torch)
    for name in ("k", "v", "score", "kind", "pos", "len"):
        getattr(other, name).copy_(getattr(steady, name))
    other.evict, steady.evict = "batched", "fused"
    assert not bench.decode_evicts_in_attention(w, other)
    for L, M in zip(steady, other):
        for name in ("q_dec", "k_dec", "v_dec"):
            getattr(M, name).copy_(getattr(L, name))
    bench.run_decode(ctx, lv, w, steady, reserve=True, step_pos=steady.steps_run + 2)
    bench.run_decode(ctx, lv, w, other, reserve=True, step_pos=steady.steps_run + 2)
    torch.cuda.synchronize()
    n = w.kv_budget
    for name in ("k", "v", "score", "kind", "pos"):
        assert torch.equal(getattr(steady, name)[:, :, :n], getattr(other, name)[:, :, :n]), name
    assert torch.equal(steady.len, other.len)
    for L, M in zip(steady, other):
        assert torch.equal(L.out_dec, M.out_dec)


def test_config4_step_in_bench_configuration():
    """Decode with the eviction inside the attention call (every cache exactly one entry over its budget)."""
    w = configs.CFG4
    ctx = lv.Context(0)
    layers, master, st = build(w)
    B = w.batch
    assert not st.groups and st.dec_bound == w.kv_budget + 1
    # the same calls without eviction on a second copy of the state give the GPU's updated score bits
    st2 = bench.StepState(w, layers, master, torch)
    for L in st2:
        ctx.decode_attn(L.q_dec, L.k_dec, L.v_dec, L.k, L.v, L.score, L.kind, L.pos, L.len, score_decay=0.9,
                        new_pos=w.seq_len, len_bound=w.kv_budget + 1, out=L.out_dec)
    torch.cuda.synchronize()
    bench.run_decode(ctx, lv, w, st, reserve=True)
    torch.cuda.synchronize()
    check = (0, 5, 13, 27)                      # layers compared entry by entry (the oracle is slow at B = 16)
    for i in check:
        sl = slice(i * B, (i + 1) * B)
        mid = snapshot(st2.k[sl], st2.v[sl], st2.score[sl], st2.kind[sl], st2.pos[sl], st2.len[sl])
        ref = O.kv_compress(*mid, mode="budget", budget=w.kv_budget, n_recent=1, order=O.ORDER_FILL)
        now = snapshot(st.k[sl], st.v[sl], st.score[sl], st.kind[sl], st.pos[sl], st.len[sl])
        same_entries(now, ref[:6])
        assert int(now[5].min()) == w.kv_budget and int(now[5].max()) == w.kv_budget
        assert torch.equal(st[i].out_dec, st2[i].out_dec)
    # and the unfused attention itself against the oracle on one layer
    i, sl = 13, slice(13 * B, 14 * B)
    st3 = bench.StepState(w, layers, master, torch)
    before = snapshot(st3.k[sl], st3.v[sl], st3.score[sl], st3.kind[sl], st3.pos[sl], st3.len[sl])
    m = master[i]
    ref = O.decode_attn(f64(m["q_dec"]), f64(m["k_dec"]), f64(m["v_dec"]), *before, score_decay=0.9,
                        new_pos=w.seq_len, out_dtype="bf16")
    assert rel_err(f64(st2[i].out_dec), ref[0]) < 2e-2
    mid = snapshot(st2.k[sl], st2.v[sl], st2.score[sl], st2.kind[sl], st2.pos[sl], st2.len[sl])
    same_entries(mid, list(ref[1:]), exact_score=False)


def test_prefill_attention_bench_mode_prints_its_line(capsys):
    """bench.py --op prefill_attn on the small fp32 configuration: the mode runs, and its JSON line carries the
    contract's fields with a roofline for the attention kernel."""
    import json
    import types
    w = configs.CFG1
    args = types.SimpleNamespace(steps=2, warmup=1, profile_steps=1, no_cpu_baseline=False)
    bench.main_prefill_attn(args, w, bench.plan(w, lv), lv.Context(0), lv, torch, DEV)
    line = [l for l in capsys.readouterr().out.splitlines() if l.startswith("{")][-1]
    out = json.loads(line)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["config"]["op"] == "prefill_attn" and out["config"]["tokens_per_layer"] == [w.seq_len]
    assert out["roofline"]["kernel"] == "prefill_attn" and out["roofline"]["achieved"] > 0
    assert out["cpu_baseline"]["kind"] == "oracle" and out["value"] > 0


def test_bench_command_line_prints_the_contract_line():
    """`python bench.py` as the driver runs it (a child process, small workload, two timed steps): exactly one JSON line on
    stdout with every field of the contract, the roofline of the dominant kernel and the oracle's CPU baseline; more than
    one GPU is refused with a message."""
    import json
    import subprocess
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "cfg1", "--steps", "2", "--warmup", "1"],
                         cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [l for l in run.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 2 and out["warmup"] == 1 and out["higher_is_better"] is True
    assert out["value"] > 0 and out["ms_per_step"] > 0 and out["vs_baseline"] is None
    assert out["config"]["workload"].startswith("cfg1") and "model" not in out["config"]
    roof = out["roofline"]
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["unit"] in ("GB/s", "TFLOP/s")
    assert roof["achieved"] > 0 and roof["peak"] > 0 and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert "traffic" in roof
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["unit"] and cpu["sample"]
    two = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT, stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True, timeout=300)
    assert two.returncode != 0 and "one GPU" in two.stderr and not two.stdout.strip()


def test_score_load_bench_mode_prints_its_table(capsys):
    """bench.py --op score_load on the one-sequence configuration: the mode runs, names the launch form the library
    takes for every row (its own decision, read back through lvlm_score_plan) and reports a positive rate."""
    import json
    import types
    w = configs.CFG2
    args = types.SimpleNamespace(steps=2, warmup=1)
    bench.main_score_load(args, w, bench.plan(w, lv), lv.Context(0), lv, torch, DEV)
    out = json.loads([l for l in capsys.readouterr().out.splitlines() if l.startswith("{")][-1])
    stages = {en["merge_to"] for en in bench.plan(w, lv) if en["merge_to"] is not None}
    assert {r["n_img"] for r in out["rows"]} == stages and len(out["rows"]) == 9 * len(stages)
    for r in out["rows"]:
        assert r["us"] > 0 and 0 < r["frac_of_peak"] < 1
        assert (r["workgroups"] is not None) == (r["form"] in ("one launch, shared tiles", "shared tiles, keys in runs"))
    assert out["value"] == max(r["TFLOPs"] for r in out["rows"])


@pytest.mark.parametrize("name", ["cfg2", "cfg4"])
def test_graph_replays_equal_the_eager_step(name):
    """The bench times HIP-graph replays of the step.  A captured (prefill, decode) pair is replayed three times on
    restored state, with eager copies and synchronisation between the replays, and every replay must leave exactly
    what the eager step leaves: caches, scores, lengths, merged hidden states, attention outputs."""
    w = configs.ALL[name]
    ctx = lv.Context(0)
    layers = bench.plan(w, lv)
    master = bench.build_master(w, layers, torch, synth, DEV)
    eager = bench.StepState(w, layers, master, torch)
    bench.run_prefill(ctx, lv, w, eager, reserve=True)
    bench.run_decode(ctx, lv, w, eager, reserve=True)
    torch.cuda.synchronize()

    st = bench.StepState(w, layers, master, torch)
    mutable = ("k", "v", "score", "kind", "pos", "len")
    saved = {n: getattr(st, n).clone() for n in mutable}
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        bench.run_prefill(ctx, lv, w, st, reserve=False)
        bench.run_decode(ctx, lv, w, st, reserve=False)
    for rep in range(3):
        for n in mutable:                                # eager work between the replays: the state goes back
            getattr(st, n).copy_(saved[n])
        for L in st:
            L.out_dec.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(st.len, eager.len), rep
        for i, (a, b) in enumerate(zip(st, eager)):
            assert torch.equal(a.out_dec, b.out_dec), (rep, i)
            if a.entry["merge_to"] is not None:
                assert torch.equal(a.hidden_out, b.hidden_out) and torch.equal(a.pos_out, b.pos_out), (rep, i)
        lens = st.len.cpu()
        for n in ("k", "v", "score", "kind", "pos"):
            x, y = getattr(st, n), getattr(eager, n)
            for row in range(0, lens.shape[0], max(1, lens.shape[0] // 7)):      # a sample of layers: whole heads
                for h in range(lens.shape[1]):
                    m = int(lens[row, h])
                    assert torch.equal(x[row, h, :m], y[row, h, :m]), (rep, n, row, h)
