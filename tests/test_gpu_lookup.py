"""GPU parity of the whole lookup and of the layer-to-layer chain, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2101_07344_amd as g
import workloads as W
from oracle import admit

from helpers import TOL, admissible_stack_inputs, compare_lookup, ideal_def, make_cache

pytestmark = pytest.mark.gpu


def _lookup_gpu(cache, act_dev, row_index, n_max, n_dev, K, want_logits=True):
    out = {
        "pred_class": torch.full((n_max,), -9, dtype=torch.int32, device="cuda"),
        "confidence": torch.full((n_max,), -9.0, device="cuda"),
        "hit": torch.full((n_max,), 77, dtype=torch.uint8, device="cuda"),
        "logits": torch.full((n_max, K), -9.0, device="cuda") if want_logits else None,
    }
    cache.lookup(act_dev, row_index, n_max, n_dev, out["pred_class"], out["confidence"], out["hit"], out["logits"])
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}


def test_tiny_config_single_cache():
    """Config 'tiny': 64 requests, fp32 [64,64,8,8], 64 -> 128 -> 10, selector 74 -> 1, tau 0.5."""
    spec = W.get_workload("tiny")
    labels, defs, weights, acts = admissible_stack_inputs(spec, calibrate_to=0.4)
    L, d, w = spec.layers[0], defs[0], weights[0]
    want = oracle.lookup(d, w, W.to_host_array(acts[0]))
    assert 0 < want["hit"].sum() < spec.batch
    cache = make_cache(g, L, w, spec.batch)
    got = _lookup_gpu(cache, acts[0].cuda(), None, spec.batch, None, L.K)
    compare_lookup(got, want, None, "f32", "tiny")
    # compacted misses
    hit_d = torch.from_numpy(got["hit"]).cuda()
    ids_out = torch.zeros(spec.batch, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    cache.compact(hit_d, None, spec.batch, None, ids_out, cnt)
    torch.cuda.synchronize()
    want_ids = oracle.compact_misses(want["hit"])
    assert int(cnt.item()) == len(want_ids)
    assert np.array_equal(ids_out.cpu().numpy()[:len(want_ids)], want_ids)
    # logits pointer NULL: same decisions, nothing else changes
    got2 = _lookup_gpu(cache, acts[0].cuda(), None, spec.batch, None, L.K, want_logits=False)
    assert np.array_equal(got2["pred_class"], got["pred_class"]) and np.array_equal(got2["confidence"], got["confidence"])
    cache.close()


STACKS = [
    # name, batch (ragged against the 32-row tiles), storage, per-layer hit target,
    # fused (gati_cache_lookup_compact) or gati_cache_lookup + gati_compact_misses
    ("resnet18", 40, "gather", 0.15, True),
    ("resnet18", 40, "gather", 0.15, False),
    ("resnet50", 37, "gather", 0.10, True),
    ("resnet50", 33, "dense", 0.20, False),
    ("bert_base", 70, "gather", 0.12, True),
    ("bert_base", 45, "dense", 0.25, True),
    ("resnet50_pool", 35, "gather", 0.12, True),       # the paper's Pool(h) predictor on the same shapes
    ("resnet50_hsel", 37, "gather", 0.12, True),       # selector network with one hidden layer
    ("resnet50_conv", 20, "gather", 0.12, True),       # the paper's Conv(k,s) predictor on the same shapes
]


@pytest.mark.parametrize("name,batch,storage,rate,fused", STACKS)
def test_stack_matches_oracle(name, batch, storage, rate, fused):
    """Every layer's class / hit / miss list bit-exact, logits and confidences within
    tolerance, with the miss counts chained on the device."""
    base = W.get_workload(name)
    spec = W.WorkloadSpec(name=f"{name}@{batch}", batch=batch, zipf_s=base.zipf_s, seed=base.seed,
                          layers=base.layers, storage=storage)
    labels, defs, weights, acts = admissible_stack_inputs(spec, calibrate_to=rate)
    host = [W.to_host_array(a) for a in acts]
    res = oracle.stack(defs, weights, host, batch, storage="gather")
    dtype = spec.layers[0].dtype
    if storage == "dense":
        dev_acts = [acts[0].cuda()] + [acts[l][torch.from_numpy(res[l - 1].ids_out.astype(np.int64))].cuda()
                                       if len(res[l - 1].ids_out) else acts[l][:1].cuda()
                                       for l in range(1, len(acts))]
    else:
        dev_acts = [a.cuda() for a in acts]
    caches = [make_cache(g, L, w, batch) for L, w in zip(spec.layers, weights)]
    stack = g.CacheStack(caches, batch, storage=storage, keep_logits=True)
    stack.run(dev_acts, fused=fused)
    torch.cuda.synchronize()
    counts = stack.counts.cpu().numpy()
    total_hits = 0
    for l, r in enumerate(res):
        n = len(r.ids_in)
        assert counts[l] == n, f"layer {l}: active count"
        assert np.array_equal(stack.ids[l].cpu().numpy()[:n], r.ids_in), f"layer {l}: ids"
        got = {"pred_class": stack.pred_class[l].cpu().numpy(), "confidence": stack.confidence[l].cpu().numpy(),
               "hit": stack.hit[l].cpu().numpy(), "logits": stack.logits[l].cpu().numpy()}
        want_ideal = None
        if dtype == "bf16" and n:
            want_ideal = oracle.lookup(ideal_def(defs[l]), weights[l], host[l], row_index=r.ids_in)
        compare_lookup(got, r.out, want_ideal, dtype, f"{spec.name} layer {l}")
        total_hits += int(r.out["hit"].sum())
    n_last = len(res[-1].ids_out)
    assert counts[len(res)] == n_last
    assert np.array_equal(stack.ids[len(res)].cpu().numpy()[:n_last], res[-1].ids_out)
    assert total_hits + n_last == batch            # every request ends in exactly one place
    assert total_hits > 0 and n_last < batch
    stack.close()


def test_resnet152_head_of_stack_dense():
    """First layers of the 50-cache streaming config (dense storage, shrinking active set)."""
    base = W.get_workload("resnet152")
    pick = [0, 3, 11, 47]            # one layer of each stage: C 256/512/1024/2048
    spec = W.WorkloadSpec(name="resnet152@24", batch=24, zipf_s=base.zipf_s, seed=base.seed,
                          layers=[base.layers[i] for i in pick], storage="dense")
    labels, defs, weights, acts = admissible_stack_inputs(spec, calibrate_to=0.3)
    host = [W.to_host_array(a) for a in acts]
    res = oracle.stack(defs, weights, host, spec.batch, storage="gather")
    dev_acts = [acts[0].cuda()] + [acts[l][torch.from_numpy(res[l - 1].ids_out.astype(np.int64))].cuda()
                                   for l in range(1, len(acts))]
    caches = [make_cache(g, L, w, spec.batch) for L, w in zip(spec.layers, weights)]
    stack = g.CacheStack(caches, spec.batch, storage="dense")
    stack.run(dev_acts)
    torch.cuda.synchronize()
    for l, r in enumerate(res):
        n = len(r.ids_in)
        assert int(stack.counts[l].item()) == n
        assert np.array_equal(stack.hit[l].cpu().numpy()[:n], r.out["hit"])
        assert np.array_equal(stack.pred_class[l].cpu().numpy()[:n], r.out["pred_class"])
        assert np.max(np.abs(stack.confidence[l].cpu().numpy()[:n] - r.out["confidence"])) <= TOL["bf16"]
    assert np.array_equal(stack.ids[4].cpu().numpy()[:len(res[-1].ids_out)], res[-1].ids_out)
    stack.close()


def test_empty_and_degenerate_active_sets():
    spec = W.get_workload("tiny")
    labels, defs, weights, acts = admissible_stack_inputs(spec)
    L = spec.layers[0]
    cache = make_cache(g, L, weights[0], spec.batch)
    act = acts[0].cuda()
    # device count 0: nothing is written
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    got = _lookup_gpu(cache, act, None, spec.batch, zero, L.K)
    assert np.all(got["pred_class"] == -9) and np.all(got["hit"] == 77) and np.all(got["logits"] == -9.0)
    # n_max = 0 is a no-op
    assert g.gati_cache_lookup(cache.handle, act, None, 0, None, None, None, None) == g.GATI_OK
    # threshold 0 -> every row hits; threshold 1 -> none (strict comparison)
    cache.set_selector(weights[0]["bs"], 0.0)
    assert np.all(_lookup_gpu(cache, act, None, spec.batch, None, L.K)["hit"] == 1)
    cache.set_selector(weights[0]["bs"], 1.0)
    assert np.all(_lookup_gpu(cache, act, None, spec.batch, None, L.K)["hit"] == 0)
    cache.set_selector(1e4, 1.0)       # sigmoid saturates to exactly 1.0f: still not above 1
    out = _lookup_gpu(cache, act, None, spec.batch, None, L.K)
    assert np.all(out["confidence"] == 1.0) and np.all(out["hit"] == 0)
    # one row, last row
    one = torch.tensor([63], dtype=torch.int32, device="cuda")
    cache.set_selector(weights[0]["bs"], L.threshold)
    got = _lookup_gpu(cache, act, one, 1, None, L.K)
    want = oracle.lookup(defs[0], weights[0], W.to_host_array(acts[0]), row_index=np.array([63], np.int32))
    compare_lookup(got, want, None, "f32", "one row")
    # fused call with nothing to look up: empty miss list
    cnt = torch.tensor([5], dtype=torch.int32, device="cuda")
    ids_out = torch.zeros(4, dtype=torch.int32, device="cuda")
    assert g.gati_cache_lookup_compact(cache.handle, act, None, 0, None, None, None, None, None, None,
                                       ids_out, cnt) == g.GATI_OK
    torch.cuda.synchronize()
    assert int(cnt.item()) == 0
    assert g.gati_cache_lookup_compact(cache.handle, act, None, 4, None, 16, 16, 16, None, None,
                                       None, cnt) == g.GATI_ERR_INVALID_ARG
    # rejected arguments leave outputs alone
    assert g.gati_cache_lookup(cache.handle, act, None, spec.batch + 1, None, 16, 16, 16) == g.GATI_ERR_INVALID_ARG
    assert g.gati_cache_lookup(cache.handle, act, None, 4, None, None, 16, 16) == g.GATI_ERR_INVALID_ARG
    cache.close()


@pytest.mark.parametrize("C,S,H,K,dtype,layout", [
    (24, 50, 40, 7, "bf16", "ncs"),       # nothing a multiple of the tile sizes
    (100, 20, 33, 33, "f32", "nsc"),      # ragged channel block, K one past a tile
    (64, 64, 64, 1500, "bf16", "ncs"),    # more classes than one pass of the head kernel holds
    (16, 16, 8, 1, "f32", "ncs"),         # one class: softmax = 1, class 0
    (72, 16, 300, 130, "f32", "ncs"),
])
def test_odd_shapes(C, S, H, K, dtype, layout):
    rng = np.random.default_rng(C + K)
    n = 45
    shape = (n, C, S) if layout == "ncs" else (n, S, C)
    x = torch.from_numpy(rng.standard_normal(shape).astype(np.float32))
    x = x.bfloat16() if dtype == "bf16" else x
    w = {"W1": (rng.standard_normal((H, C)) * np.sqrt(2 / C)).astype(np.float32),
         "b1": (rng.standard_normal(H) * 0.1).astype(np.float32),
         "W2": (rng.standard_normal((K, H)) * np.sqrt(2 / H)).astype(np.float32),
         "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
         "ws": (rng.standard_normal(C + K) * 0.5).astype(np.float32), "bs": 0.1}
    d = oracle.CacheDef(C=C, S=S, H=H, K=K, dtype=dtype, layout=layout, threshold=0.5,
                        round_operands=(dtype == "bf16"))
    host = W.to_host_array(x)
    ok = np.setdiff1d(np.arange(n), admit.inadmissible_rows(d, w, host)).astype(np.int32)
    assert len(ok) > n // 2
    want = oracle.lookup(d, w, host, row_index=ok)
    cache = g.Cache(C, S, H, K, dtype, layout, 0.5, n, w)
    got = _lookup_gpu(cache, x.cuda(), torch.from_numpy(ok).cuda(), len(ok), None, K)
    want_ideal = oracle.lookup(ideal_def(d), w, host, row_index=ok) if dtype == "bf16" else None
    compare_lookup(got, want, want_ideal, dtype, f"odd {C}x{S}x{H}x{K}")
    cache.close()


@pytest.mark.parametrize("dtype,K", [("f32", 10), ("bf16", 1000)])
def test_softmax_threshold_selector(dtype, K):
    """No selector network: hit iff the top class probability exceeds the threshold."""
    rng = np.random.default_rng(K)
    n, C, S, H = 70, 128, 49, 96
    x = torch.from_numpy(np.maximum(rng.standard_normal((n, C, S)) + 0.3, 0).astype(np.float32))
    x = x.bfloat16() if dtype == "bf16" else x
    w = {"W1": (rng.standard_normal((H, C)) * np.sqrt(2 / C)).astype(np.float32), "b1": np.zeros(H, np.float32),
         "W2": (rng.standard_normal((K, H)) * np.sqrt(2 / H)).astype(np.float32), "b2": np.zeros(K, np.float32),
         "ws": (rng.standard_normal(C + K) * 3).astype(np.float32), "bs": 2.0}
    host = W.to_host_array(x)
    probe = oracle.CacheDef(C=C, S=S, H=H, K=K, dtype=dtype, threshold=0.0, round_operands=(dtype == "bf16"),
                            selector="softmax")
    tau = float(np.float32(np.median(oracle.lookup(probe, w, host)["confidence"])))   # about half the rows hit
    d = oracle.CacheDef(C=C, S=S, H=H, K=K, dtype=dtype, threshold=tau, round_operands=(dtype == "bf16"),
                        selector="softmax")
    ok = np.setdiff1d(np.arange(n), admit.inadmissible_rows(d, w, host)).astype(np.int32)
    want = oracle.lookup(d, w, host, row_index=ok)
    assert 0 < want["hit"].sum() < len(ok)
    cache = g.Cache(C, S, H, K, dtype, "ncs", tau, n, w, selector="softmax")
    got = _lookup_gpu(cache, x.cuda(), torch.from_numpy(ok).cuda(), len(ok), None, K)
    want_ideal = oracle.lookup(ideal_def(d), w, host, row_index=ok) if dtype == "bf16" else None
    compare_lookup(got, want, want_ideal, dtype, f"softmax selector {dtype}")
    cache.close()
    # the mode reads no selector weights: a cache built without them gives the same bits
    bare = g.Cache(C, S, H, K, dtype, "ncs", tau, n, {k: v for k, v in w.items() if k not in ("ws", "bs")}, selector="softmax")
    got2 = _lookup_gpu(bare, x.cuda(), torch.from_numpy(ok).cuda(), len(ok), None, K)
    for key in ("pred_class", "confidence", "hit", "logits"):
        assert np.array_equal(got[key][:len(ok)], got2[key][:len(ok)]), key
    bare.close()


@pytest.mark.parametrize("dtype,predictor,K,Hs,want_logits", [
    ("f32", "gap_mlp", 10, 8, True),        # fp32 MFMA first layer, one partial tile of units
    ("bf16", "gap_mlp", 1000, 64, False),   # probabilities from the library's own logits buffer
    ("bf16", "pool_fc", 100, 33, True),     # features = ReLU'd window means
    ("bf16", "fc_mlp", 37, 130, True),      # features = the FC(h) hidden layer
])
def test_hidden_layer_selector(dtype, predictor, K, Hs, want_logits):
    """Selector network with one hidden layer over [features ; class probabilities]."""
    rng = np.random.default_rng(K + Hs)
    n, C, ih, iw, H = 90, 32, 8, 8, 96
    S = ih * iw
    kw = dict(predictor=predictor)
    if predictor == "pool_fc":
        kw.update(in_hw=(ih, iw), out_hw=(2, 2))
    d0 = oracle.CacheDef(C=C, S=S, H=0 if predictor == "pool_fc" else H, K=K, dtype=dtype, threshold=0.5,
                         round_operands=(dtype == "bf16"), selector="hidden", sel_hidden=Hs, **kw)
    F = d0.F
    x = torch.from_numpy(np.maximum(rng.standard_normal((n, C, S)) + 0.3, 0).astype(np.float32))
    x = x.bfloat16() if dtype == "bf16" else x
    fan1 = C * S if predictor == "fc_mlp" else C
    Hin = F if predictor == "pool_fc" else H
    w = {"W1": (rng.standard_normal((H, fan1)) * np.sqrt(2 / fan1)).astype(np.float32), "b1": np.zeros(H, np.float32),
         "W2": (rng.standard_normal((K, Hin)) * np.sqrt(2 / Hin)).astype(np.float32),
         "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
         "Ws": (rng.standard_normal((Hs, F + K)) * 4 * np.sqrt(2 / (F + K))).astype(np.float32),
         "cs": (rng.standard_normal(Hs) * 0.1).astype(np.float32),
         "vs": (rng.standard_normal(Hs) * np.sqrt(2 / Hs)).astype(np.float32), "bs": 0.0}
    host = W.to_host_array(x)
    s0 = oracle.lookup(d0, w, host)["score"]
    w["bs"] = float(np.float32(-np.median(s0)))          # about half the rows hit
    ok = np.setdiff1d(np.arange(n), admit.inadmissible_rows(d0, w, host)).astype(np.int32)
    assert len(ok) > n // 2
    want = oracle.lookup(d0, w, host, row_index=ok)
    assert 0 < want["hit"].sum() < len(ok)
    cache = g.Cache(C, S, d0.H, K, dtype, "ncs", 0.5, n, w, selector="hidden", sel_hidden=Hs,
                    in_hw=kw.get("in_hw", (0, 0)), out_hw=kw.get("out_hw", (0, 0)), predictor=predictor)
    m = len(ok)
    okd = torch.from_numpy(ok).cuda()
    got = _lookup_gpu(cache, x.cuda(), okd, m, None, K, want_logits=want_logits)
    want_ideal = oracle.lookup(ideal_def(d0), w, host, row_index=ok) if dtype == "bf16" else None
    compare_lookup(got, want, want_ideal, dtype, f"hidden selector {dtype} {predictor}",
                   tol_ideal=5e-2 if predictor == "fc_mlp" else None)
    # fused compaction gives the same flags and the oracle's miss list
    out = {"pred_class": torch.zeros(m, dtype=torch.int32, device="cuda"), "confidence": torch.zeros(m, device="cuda"),
           "hit": torch.zeros(m, dtype=torch.uint8, device="cuda")}
    ids_out = torch.zeros(m, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    cache.lookup_compact(x.cuda(), okd, m, None, out["pred_class"], out["confidence"], out["hit"], None,
                         okd, ids_out, cnt)
    torch.cuda.synchronize()
    assert np.array_equal(out["hit"].cpu().numpy(), got["hit"]) and \
        np.array_equal(out["confidence"].cpu().numpy(), got["confidence"])
    want_ids = oracle.compact_misses(want["hit"], ok)
    assert int(cnt.item()) == len(want_ids) and np.array_equal(ids_out.cpu().numpy()[:len(want_ids)], want_ids)
    cache.close()


@pytest.mark.parametrize("predictor,selector", [("gap_mlp", "linear"), ("gap_mlp", "hidden"), ("pool_fc", "linear"),
                                                ("fc_mlp", "linear"), ("conv_fc", "linear")])
def test_set_weights_swaps_in_a_retrained_cache(predictor, selector):
    """Weights replaced in place (the paper's periodic cache replacement) behave exactly like a cache
    created with them, and the lookup follows the oracle before and after."""
    n, C, hw, H, K, Hs = 48, 32, 8, 24, 11, 9
    S = hw * hw
    kw = dict(predictor=predictor)
    if predictor == "pool_fc":
        kw.update(in_hw=(hw, hw), out_hw=(2, 2))
    if predictor == "conv_fc":
        kw.update(in_hw=(hw, hw), conv_ks=(3, 1))
        H = 4
    d = oracle.CacheDef(C=C, S=S, H=0 if predictor == "pool_fc" else H, K=K, dtype="bf16", threshold=0.5, round_operands=True,
                        selector=selector, sel_hidden=Hs if selector == "hidden" else 0, **kw)
    F = d.F
    rng = np.random.default_rng(len(predictor) + len(selector))
    x = torch.from_numpy(np.maximum(rng.standard_normal((n, C, S)) + 0.3, 0).astype(np.float32)).bfloat16()
    host = W.to_host_array(x)

    def draw():
        fan1 = {"fc_mlp": C * S, "conv_fc": C * 9}.get(predictor, C)
        shape1 = (H, C, 3, 3) if predictor == "conv_fc" else (H, fan1)
        Hin = F if predictor in ("pool_fc", "conv_fc") else H
        w = {"W1": (rng.standard_normal(shape1) * np.sqrt(2 / fan1)).astype(np.float32),
             "b1": (rng.standard_normal(H) * 0.1).astype(np.float32),
             "W2": (rng.standard_normal((K, Hin)) * np.sqrt(2 / Hin)).astype(np.float32),
             "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
             "ws": (rng.standard_normal(F + K) * 2 * np.sqrt(2 / (F + K))).astype(np.float32), "bs": 0.0}
        if selector == "hidden":
            w.update(Ws=(rng.standard_normal((Hs, F + K)) * 4 * np.sqrt(2 / (F + K))).astype(np.float32),
                     cs=(rng.standard_normal(Hs) * 0.1).astype(np.float32),
                     vs=(rng.standard_normal(Hs) * np.sqrt(2 / Hs)).astype(np.float32))
        w["bs"] = float(np.float32(-np.median(oracle.lookup(d, w, host)["score"])))
        return w

    wa, wb = draw(), draw()
    mk = lambda w: g.Cache(C, S, d.H, K, "bf16", "ncs", 0.5, n, w, selector=selector, predictor=predictor,
                           in_hw=kw.get("in_hw", (0, 0)), out_hw=kw.get("out_hw", (0, 0)),
                           sel_hidden=d.sel_hidden, conv_ks=kw.get("conv_ks", (0, 0)))
    cache, fresh_b = mk(wa), mk(wb)
    xd = x.cuda()
    for w_now, other in ((wa, None), (wb, fresh_b)):
        if other is not None:
            cache.set_weights(w_now)
        ok = np.setdiff1d(np.arange(n), admit.inadmissible_rows(d, w_now, host)).astype(np.int32)
        okd = torch.from_numpy(ok).cuda()
        got = _lookup_gpu(cache, xd, okd, len(ok), None, K)
        want = oracle.lookup(d, w_now, host, row_index=ok)
        compare_lookup(got, want, None, "bf16", f"set_weights {predictor}/{selector}")
        if other is not None:
            ref = _lookup_gpu(other, xd, okd, len(ok), None, K)
            for key in ("pred_class", "confidence", "hit", "logits"):
                assert np.array_equal(got[key], ref[key]), key       # bit for bit the cache created with them
    assert not np.array_equal(oracle.lookup(d, wa, host)["pred_class"], oracle.lookup(d, wb, host)["pred_class"])
    cache.close()
    fresh_b.close()
