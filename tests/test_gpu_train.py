"""GPU parity of the retraining step (Section 3, "Training Learned Caches"; Section 5, "Retraining
Learned Caches") against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2101_07344_amd as g
import workloads as W
from oracle import admit, train

pytestmark = pytest.mark.gpu

# fp32 sums of up to 2048 products against fp64: a gradient entry is good to 1e-4 of the largest
# entry of its tensor (the same bar as the lookup's logits); the update theta - lr*g adds half an
# ulp of theta.
G_RTOL, ULP = 1e-4, 1.2e-7
PARAMS = ("W1", "b1", "W2", "b2", "ws")


def _inputs(name, layer, n):
    base = W.get_workload(name)
    spec = W.WorkloadSpec(name=f"{name}@{n}", batch=n, zipf_s=base.zipf_s, seed=base.seed + 11,
                          layers=base.layers[layer:layer + 1], storage="gather")
    L = spec.layers[0]
    labels = W.zipf_labels(n, L.K, spec.zipf_s, spec.seed)
    w = W.cache_weights(spec, 0)
    act = W.activation_bulk(spec, 0, labels, np.arange(n), device="cpu")
    Y = W.teacher_distribution(labels, L.K, spec.seed)
    d = admit.cache_defs(spec, mirror=False)[0]
    pooled_ref = oracle.pool(d, W.to_host_array(act))
    return spec, L, labels, w, act, Y, pooled_ref


def _gpu_pooled(L, w, act, n):
    cache = g.Cache.from_layer(L, w, n)
    pooled = torch.empty((n, L.C), device="cuda")
    cache.pool(act.cuda(), None, n, None, pooled)
    torch.cuda.synchronize()
    return cache, pooled


def _margin_ok(w, pooled_ref, Y):
    """The selector's ground truth compares two argmaxes: the logits' top-2 gap must be far above
    fp32 rounding for both sides to take the same decision."""
    z = np.sort(train.forward(w, pooled_ref)["z"], axis=1)
    ys = np.sort(Y.astype(np.float64), axis=1)
    return (z[:, -1] - z[:, -2]).min() > 1e-5 and (ys[:, -1] - ys[:, -2]).min() > 0


def _check_update(got, want, old, grads, lr, steps=1, where=""):
    for k in [k for k in want if k != "bs"]:
        tol = steps * (lr * G_RTOL * np.max(np.abs(grads[k])) + ULP * np.max(np.abs(old[k])))
        err = np.max(np.abs(got[k].astype(np.float64) - want[k]))
        assert err <= tol, f"{where}: {k} max abs err {err} > {tol}"
    tol = steps * (lr * G_RTOL * abs(grads["bs"]) + ULP * max(abs(old["bs"]), 1e-3))
    assert abs(got["bs"] - want["bs"]) <= tol, f"{where}: bs {got['bs']} vs {want['bs']}"


CASES = [("tiny", 0, 64), ("tiny", 0, 37), ("tiny", 0, 1), ("resnet18", 4, 100), ("resnet18", 7, 130),
         ("resnet50", 3, 96), ("resnet50", 13, 70), ("bert_base", 0, 149)]


@pytest.mark.parametrize("name,layer,n", CASES)
@pytest.mark.parametrize("lr,alpha,lam", [(1.0, 0.3, 2.0)])
def test_one_step_gradients(name, layer, n, lr, alpha, lam):
    """lr = 1 turns the weight change into the gradient itself."""
    spec, L, labels, w, act, Y, pooled_ref = _inputs(name, layer, n)
    assert _margin_ok(w, pooled_ref, Y)
    cache, pooled = _gpu_pooled(L, w, act, n)
    assert np.max(np.abs(pooled.cpu().numpy() - pooled_ref)) <= 2e-6 * max(1.0, np.max(np.abs(pooled_ref)))
    tr = g.Trainer(L.C, L.H, L.K, w, max_rows=n + 3)
    losses = torch.full((2,), -1.0, device="cuda")
    tr.step(pooled, torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda(), lr, alpha, lam, losses)
    torch.cuda.synchronize()
    got = tr.get_weights()
    want, lp, ls = train.sgd_step(w, pooled_ref, labels, Y, lr, alpha, lam)
    grads = train.gradients(w, pooled_ref, labels, Y, alpha, lam)
    _check_update(got, want, w, grads, lr, where=f"{name}[{layer}] n={n}")
    lg = losses.cpu().numpy()
    assert abs(lg[0] - lp) <= 1e-5 * max(1.0, abs(lp)) and abs(lg[1] - ls) <= 1e-5 * max(1.0, abs(ls)), (lg, lp, ls)
    tr.close(); cache.close()


@pytest.mark.parametrize("name,layer,n", [("tiny", 0, 64), ("resnet18", 6, 120), ("resnet50", 9, 200)])
def test_five_steps_then_serve(name, layer, n):
    """The paper's retraining parameters (Section 7: learning rate 0.002, 5 epochs) on one batch,
    then the retrained weights go into a serving cache whose lookups match the oracle's lookups
    under the oracle-trained weights."""
    lr, alpha, lam = 0.002, 0.5, 3.0
    spec, L, labels, w, act, Y, pooled_ref = _inputs(name, layer, n)
    cache, pooled = _gpu_pooled(L, w, act, n)
    tr = g.Trainer(L.C, L.H, L.K, w, max_rows=n)
    lab_d, Y_d = torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda()
    losses = torch.zeros((5, 2), device="cuda")
    cur, want_losses, gmax = w, [], None
    for e in range(5):
        assert _margin_ok(cur, pooled_ref, Y)
        tr.step(pooled, lab_d, Y_d, lr, alpha, lam, losses[e])
        grads = train.gradients(cur, pooled_ref, labels, Y, alpha, lam)
        gmax = grads if gmax is None else {k: np.maximum(np.abs(gmax[k]), np.abs(grads[k])) for k in grads}
        cur, lp, ls = train.sgd_step(cur, pooled_ref, labels, Y, lr, alpha, lam)
        want_losses.append((lp, ls))
    torch.cuda.synchronize()
    got = tr.get_weights()
    _check_update(got, cur, w, gmax, lr, steps=5, where=f"{name}[{layer}] 5 steps")
    assert np.allclose(losses.cpu().numpy(), np.array(want_losses), rtol=2e-5, atol=1e-6)
    assert want_losses[-1][0] < want_losses[0][0]            # it learns
    # serve with the retrained weights
    cache.set_weights(got)
    d = admit.cache_defs(spec, mirror=False)[0]
    w64 = {k: (np.asarray(v, np.float32) if k != "bs" else float(np.float32(v))) for k, v in cur.items()}
    want = oracle.lookup(d, w64, W.to_host_array(act))
    pc = torch.empty(n, dtype=torch.int32, device="cuda")
    conf = torch.empty(n, device="cuda")
    hit = torch.empty(n, dtype=torch.uint8, device="cuda")
    logits = torch.empty((n, L.K), device="cuda")
    cache.lookup(act.cuda(), None, n, None, pc, conf, hit, logits)
    torch.cuda.synchronize()
    tol = 1e-4 if L.dtype == "f32" else 2e-2
    assert np.max(np.abs(logits.cpu().numpy() - want["logits"])) <= tol
    assert np.max(np.abs(conf.cpu().numpy() - want["confidence"])) <= tol
    z = np.sort(want["logits"].astype(np.float64), axis=1)
    clear = (z[:, -1] - z[:, -2]) > 10 * tol
    assert np.array_equal(pc.cpu().numpy()[clear], want["pred_class"][clear])
    tr.close(); cache.close()


@pytest.mark.parametrize("C,H,K,n", [(40, 24, 100, 19), (37, 50, 1100, 23), (130, 65, 7, 70), (64, 33, 257, 5)])
def test_odd_shapes_cover_every_kernel_path(C, H, K, n):
    """Sizes that are multiples of nothing: scalar operand loads (leading dimensions not multiples
    of 4), ragged 64 x 64 tiles, and the row kernel's four class-count ranges (K <= 64, <= 256,
    <= 1024, larger)."""
    rng = np.random.default_rng(C * 1000 + K)
    w = {"W1": (rng.standard_normal((H, C)) * np.sqrt(2.0 / C)).astype(np.float32),
         "b1": (rng.standard_normal(H) * 0.1).astype(np.float32),
         "W2": (rng.standard_normal((K, H)) * np.sqrt(2.0 / H)).astype(np.float32),
         "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
         "ws": (rng.standard_normal(C + K) * 0.3).astype(np.float32), "bs": 0.25}
    pooled = rng.standard_normal((n, C)).astype(np.float32)
    labels = rng.integers(0, K, n).astype(np.int32)
    Y = W.teacher_distribution(labels, K, seed=K)
    assert _margin_ok(w, pooled, Y)
    lr, alpha, lam = 1.0, 0.6, 1.5
    tr = g.Trainer(C, H, K, w, max_rows=n)
    losses = torch.zeros(2, device="cuda")
    tr.step(torch.from_numpy(pooled).cuda(), torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda(),
            lr, alpha, lam, losses)
    torch.cuda.synchronize()
    want, lp, ls = train.sgd_step(w, pooled, labels, Y, lr, alpha, lam)
    grads = train.gradients(w, pooled, labels, Y, alpha, lam)
    _check_update(tr.get_weights(), want, w, grads, lr, where=f"C={C} H={H} K={K} n={n}")
    lg = losses.cpu().numpy()
    assert abs(lg[0] - lp) <= 1e-5 * max(1.0, abs(lp)) and abs(lg[1] - ls) <= 1e-5 * max(1.0, abs(ls))
    tr.close()


def _hidden_case(C, H, K, Hs, n, seed):
    rng = np.random.default_rng(seed)
    w = {"W1": (rng.standard_normal((H, C)) * np.sqrt(2.0 / C)).astype(np.float32),
         "b1": (rng.standard_normal(H) * 0.1).astype(np.float32),
         "W2": (rng.standard_normal((K, H)) * np.sqrt(2.0 / H)).astype(np.float32),
         "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
         "Ws": (rng.standard_normal((Hs, C + K)) * np.sqrt(2.0 / (C + K))).astype(np.float32),
         "cs": (rng.standard_normal(Hs) * 0.2).astype(np.float32),
         "vs": (rng.standard_normal(Hs) * 0.5).astype(np.float32), "bs": -0.1}
    pooled = rng.standard_normal((n, C)).astype(np.float32)
    labels = rng.integers(0, K, n).astype(np.int32)
    return w, pooled, labels, W.teacher_distribution(labels, K, seed=seed)


@pytest.mark.parametrize("C,H,K,Hs,n", [(64, 32, 10, 16, 40), (37, 20, 50, 33, 21), (256, 128, 1000, 64, 131),
                                        (96, 48, 300, 70, 65)])
def test_hidden_layer_selector_step(C, H, K, Hs, n):
    """The paper's selector shape (Section 3, "Selector Network Design"): gradients with lr = 1, then
    three more steps at a small rate."""
    w, pooled, labels, Y = _hidden_case(C, H, K, Hs, n, seed=C + Hs)
    assert _margin_ok(w, pooled, Y)
    f = train.forward(w, pooled)
    assert np.min(np.abs(f["sa"])) > 1e-6            # no hidden unit sits on the ReLU's kink
    pd, ld, Yd = torch.from_numpy(pooled).cuda(), torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda()
    tr = g.Trainer(C, H, K, w, max_rows=n, sel_hidden=Hs)
    losses = torch.zeros(2, device="cuda")
    tr.step(pd, ld, Yd, 1.0, 0.3, 2.0, losses)
    torch.cuda.synchronize()
    want, lp, ls = train.sgd_step(w, pooled, labels, Y, 1.0, 0.3, 2.0)
    grads = train.gradients(w, pooled, labels, Y, 0.3, 2.0)
    got = tr.get_weights()
    assert set(got) == set(want)
    _check_update(got, want, w, grads, 1.0, where=f"hidden selector C={C} Hs={Hs}")
    lg = losses.cpu().numpy()
    assert abs(lg[0] - lp) <= 1e-5 * max(1.0, abs(lp)) and abs(lg[1] - ls) <= 1e-5 * max(1.0, abs(ls)), (lg, lp, ls)
    tr.close()
    # a fresh trainer, four steps at a small rate
    tr = g.Trainer(C, H, K, w, max_rows=n + 5, sel_hidden=Hs)
    cur, gmax = w, None
    for _ in range(4):
        fc = train.forward(cur, pooled)
        assert _margin_ok(cur, pooled, Y) and np.min(np.abs(fc["sa"])) > 1e-6
        tr.step(pd, ld, Yd, 0.01, 0.5, 3.0)
        gr = train.gradients(cur, pooled, labels, Y, 0.5, 3.0)
        gmax = gr if gmax is None else {k: np.maximum(np.abs(gmax[k]), np.abs(gr[k])) for k in gr}
        cur, _, _ = train.sgd_step(cur, pooled, labels, Y, 0.01, 0.5, 3.0)
    torch.cuda.synchronize()
    _check_update(tr.get_weights(), cur, w, gmax, 0.01, steps=4, where="hidden selector, 4 steps")
    tr.close()


def test_hidden_selector_retrain_then_serve():
    """Retrain a resnet50_hsel cache's predictor and hidden-layer selector, swap the weights into the
    serving cache, and look up."""
    base = W.get_workload("resnet50_hsel")
    n = 96
    spec = W.WorkloadSpec(name="hsel@96", batch=n, zipf_s=base.zipf_s, seed=base.seed + 3, layers=base.layers[8:9],
                          storage="gather")
    L = spec.layers[0]
    labels = W.zipf_labels(n, L.K, spec.zipf_s, spec.seed)
    w = W.cache_weights(spec, 0)
    act = W.activation_bulk(spec, 0, labels, np.arange(n), device="cpu")
    Y = W.teacher_distribution(labels, L.K, spec.seed)
    d = admit.cache_defs(spec, mirror=False)[0]
    pooled_ref = oracle.pool(d, W.to_host_array(act))
    cache, pooled = _gpu_pooled(L, w, act, n)
    tr = g.Trainer(L.C, L.H, L.K, w, max_rows=n, sel_hidden=L.sel_hidden)
    cur = {k: w[k] for k in ("W1", "b1", "W2", "b2", "Ws", "cs", "vs", "bs")}
    for _ in range(3):
        assert _margin_ok(cur, pooled_ref, Y)
        tr.step(pooled, torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda(), 0.002, 0.5, 2.0)
        cur, _, _ = train.sgd_step(cur, pooled_ref, labels, Y, 0.002, 0.5, 2.0)
    torch.cuda.synchronize()
    got = tr.get_weights()
    cache.set_weights(got)
    w32 = {k: (np.asarray(v, np.float32) if k != "bs" else float(np.float32(v))) for k, v in cur.items()}
    want = oracle.lookup(d, w32, W.to_host_array(act))
    pc = torch.empty(n, dtype=torch.int32, device="cuda")
    conf = torch.empty(n, device="cuda")
    hit = torch.empty(n, dtype=torch.uint8, device="cuda")
    logits = torch.empty((n, L.K), device="cuda")
    cache.lookup(act.cuda(), None, n, None, pc, conf, hit, logits)
    torch.cuda.synchronize()
    assert np.max(np.abs(logits.cpu().numpy() - want["logits"])) <= 2e-2
    assert np.max(np.abs(conf.cpu().numpy() - want["confidence"])) <= 2e-2
    tr.close(); cache.close()


@pytest.mark.parametrize("layer,n,sel_hidden", [(3, 64, 0), (13, 50, 0), (8, 40, 24)])
def test_pool_fc_predictor_step(layer, n, sel_hidden):
    """The paper's Pool(h) predictor (no hidden layer): features from gati_cache_pool of a Pool(h)
    cache, one step with lr = 1, then the retrained weights serve lookups."""
    base = W.get_workload("resnet50_pool")
    spec = W.WorkloadSpec(name=f"pool@{n}", batch=n, zipf_s=base.zipf_s, seed=base.seed + 5,
                          layers=base.layers[layer:layer + 1], storage="gather")
    L = spec.layers[0]
    labels = W.zipf_labels(n, L.K, spec.zipf_s, spec.seed)
    w = W.cache_weights(spec, 0)
    act = W.activation_bulk(spec, 0, labels, np.arange(n), device="cpu")
    Y = W.teacher_distribution(labels, L.K, spec.seed)
    d = admit.cache_defs(spec, mirror=False)[0]
    feats_ref = oracle.pool(d, W.to_host_array(act))
    F = feats_ref.shape[1]
    wt = {"W2": w["W2"], "b2": w["b2"], "bs": w["bs"]}
    if sel_hidden:
        rng = np.random.default_rng(layer)
        wt.update({"Ws": (rng.standard_normal((sel_hidden, F + L.K)) * np.sqrt(2.0 / (F + L.K))).astype(np.float32),
                   "cs": (rng.standard_normal(sel_hidden) * 0.2).astype(np.float32),
                   "vs": (rng.standard_normal(sel_hidden) * 0.5).astype(np.float32)})
    else:
        wt["ws"] = w["ws"]
    assert _margin_ok(wt, feats_ref, Y)
    cache = g.Cache.from_layer(L, w, n)
    feats = torch.empty((n, F), device="cuda")
    cache.pool(act.cuda(), None, n, None, feats)
    tr = g.Trainer(L.C, 0, L.K, wt, max_rows=n, sel_hidden=sel_hidden, predictor="pool_fc", out_hw=L.out_hw)
    losses = torch.zeros(2, device="cuda")
    tr.step(feats, torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda(), 1.0, 0.4, 2.0, losses)
    torch.cuda.synchronize()
    got = tr.get_weights()
    want, lp, ls = train.sgd_step(wt, feats_ref, labels, Y, 1.0, 0.4, 2.0)
    grads = train.gradients(wt, feats_ref, labels, Y, 0.4, 2.0)
    assert set(got) == set(want)
    _check_update(got, want, wt, grads, 1.0, where=f"pool_fc layer {layer}")
    lg = losses.cpu().numpy()
    assert abs(lg[0] - lp) <= 1e-5 * max(1.0, abs(lp)) and abs(lg[1] - ls) <= 1e-5 * max(1.0, abs(ls))
    tr.close(); cache.close()


def test_minibatch_epochs():
    """Two epochs over 150 samples in batches of 64 (64 + 64 + 22): sliced inputs, ragged last batch."""
    lr, alpha, lam = 0.01, 0.4, 2.0
    spec, L, labels, w, act, Y, pooled_ref = _inputs("resnet18", 5, 150)
    cache, pooled = _gpu_pooled(L, w, act, 150)
    tr = g.Trainer(L.C, L.H, L.K, w, max_rows=64)
    losses = torch.zeros((2, 3, 2), device="cuda")
    tr.fit(pooled, torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda(), 2, 64, lr, alpha, lam, losses)
    cur, want, gmax = w, [], None
    for e in range(2):
        for lo in range(0, 150, 64):
            sl = slice(lo, min(150, lo + 64))
            assert _margin_ok(cur, pooled_ref[sl], Y[sl])
            grads = train.gradients(cur, pooled_ref[sl], labels[sl], Y[sl], alpha, lam)
            gmax = grads if gmax is None else {k: np.maximum(np.abs(gmax[k]), np.abs(grads[k])) for k in grads}
            cur, lp, ls = train.sgd_step(cur, pooled_ref[sl], labels[sl], Y[sl], lr, alpha, lam)
            want.append((lp, ls))
    torch.cuda.synchronize()
    _check_update(tr.get_weights(), cur, w, gmax, lr, steps=6, where="minibatch epochs")
    assert np.allclose(losses.cpu().numpy().reshape(6, 2), np.array(want), rtol=2e-5, atol=1e-6)
    tr.close(); cache.close()


def test_steps_are_bit_reproducible():
    """No float atomics, every reduction in a fixed order: two trainers fed the same three steps end
    with identical bits, for both selectors."""
    for hid in (0, 16):
        if hid:
            w, pooled, labels, Y = _hidden_case(72, 40, 130, hid, 90, seed=9)
        else:
            spec, L, labels, w, act, Y, pooled = _inputs("resnet18", 6, 90)
        C, H, K = w["W1"].shape[1], w["W1"].shape[0], w["W2"].shape[0]
        pd, ld, Yd = torch.from_numpy(np.ascontiguousarray(pooled)).cuda(), torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda()
        outs = []
        for _ in range(2):
            tr = g.Trainer(C, H, K, w, max_rows=90, sel_hidden=hid)
            losses = torch.zeros((3, 2), device="cuda")
            for s in range(3):
                tr.step(pd, ld, Yd, 0.05, 0.5, 2.0, losses[s])
            torch.cuda.synchronize()
            outs.append((tr.get_weights(), losses.cpu().numpy()))
            tr.close()
        for k in outs[0][0]:
            assert np.array_equal(np.asarray(outs[0][0][k]), np.asarray(outs[1][0][k])), k
        assert np.array_equal(outs[0][1], outs[1][1])


def test_step_replays_from_a_hip_graph():
    """The step only enqueues kernels, so a serving loop can capture it: three replays of one captured
    step leave the same weights, bit for bit, as three eager steps."""
    spec, L, labels, w, act, Y, pooled = _inputs("resnet18", 5, 100)
    pd, ld, Yd = torch.from_numpy(np.ascontiguousarray(pooled)).cuda(), torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda()
    eager = g.Trainer(L.C, L.H, L.K, w, max_rows=100)
    for _ in range(3):
        eager.step(pd, ld, Yd, 0.01, 0.5, 2.0)
    torch.cuda.synchronize()
    want = eager.get_weights()
    eager.close()
    tr = g.Trainer(L.C, L.H, L.K, w, max_rows=100)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    losses = torch.zeros(2, device="cuda")
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            tr.step(pd, ld, Yd, 0.01, 0.5, 2.0, losses)          # captured, not run
    for _ in range(3):
        junk = torch.randn(64, 64, device="cuda") @ torch.randn(64, 64, device="cuda")
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
    got = tr.get_weights()
    for k in want:
        assert np.array_equal(np.asarray(got[k]), np.asarray(want[k])), k
    assert torch.isfinite(junk).all() and float(losses[0]) > 0
    tr.close()


def test_step_argument_checks_and_empty_batch():
    spec, L, labels, w, act, Y, pooled_ref = _inputs("tiny", 0, 8)
    tr = g.Trainer(L.C, L.H, L.K, w, max_rows=8)
    pooled = torch.from_numpy(pooled_ref).cuda()
    lab, Yd = torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda()
    p = g.TrainParams(0.1, 0.5, 2.0)
    assert g.gati_trainer_step(tr.handle, pooled, L.C, 9, lab, Yd, L.K, p) == g.GATI_ERR_INVALID_ARG     # n > max_rows
    assert g.gati_trainer_step(tr.handle, pooled, L.C - 1, 8, lab, Yd, L.K, p) == g.GATI_ERR_INVALID_ARG
    assert g.gati_trainer_step(tr.handle, None, L.C, 8, lab, Yd, L.K, p) == g.GATI_ERR_INVALID_ARG
    assert g.gati_trainer_step(tr.handle, pooled, L.C, 8, lab, Yd, L.K, g.TrainParams(0.1, 1.5, 2.0)) == g.GATI_ERR_INVALID_ARG
    assert g.gati_trainer_step(tr.handle, pooled, L.C, 0, None, None, L.K, p) == g.GATI_OK               # empty: no-op
    torch.cuda.synchronize()
    got = tr.get_weights()
    assert all(np.array_equal(got[k], w[k]) for k in PARAMS) and got["bs"] == float(np.float32(w["bs"]))
    tr.close()


def _simplex(rng, n, K):
    Y = rng.random((n, K)).astype(np.float32) + 0.05
    return Y / Y.sum(axis=1, keepdims=True, dtype=np.float32)


def _w32(w):
    return {k: (np.asarray(v, np.float32) if k != "bs" else float(v)) for k, v in w.items()}


@pytest.mark.parametrize("C,S,H,K,n,selector", [
    (8, 16, 40, 7, 45, "linear"), (3, 50, 33, 12, 30, "linear"), (16, 49, 64, 100, 70, "hidden"), (6, 20, 24, 9, 33, "softmax"),
])
def test_fc_predictor_step(C, S, H, K, n, selector):
    """FC(h): the first layer reads the flattened row; the selector reads [h ; q] as data."""
    rng = np.random.default_rng(C * S + H)
    D = C * S
    w = {"W1": rng.standard_normal((H, D)) * np.sqrt(2.0 / D), "b1": rng.standard_normal(H) * 0.1,
         "W2": rng.standard_normal((K, H)) * np.sqrt(2.0 / H), "b2": rng.standard_normal(K) * 0.1}
    if selector == "linear":
        w.update({"ws": rng.standard_normal(H + K) * 0.3, "bs": 0.2})
    elif selector == "hidden":
        w.update({"Ws": rng.standard_normal((10, H + K)) * 0.3, "cs": rng.standard_normal(10) * 0.1,
                  "vs": rng.standard_normal(10) * 0.5, "bs": 0.2})
    w = _w32(w)
    x = np.maximum(rng.standard_normal((n, D)), 0).astype(np.float32)
    labels = rng.integers(0, K, n).astype(np.int32)
    Y = _simplex(rng, n, K)
    arch = {"sel_input": "hidden"}
    z = np.sort(train.forward(w, x, arch)["z"], axis=1)
    assert (z[:, -1] - z[:, -2]).min() > 1e-5
    tr = g.Trainer(C, H, K, w, max_rows=n, predictor="fc_mlp", S=S, selector=selector, sel_hidden=10 if selector == "hidden" else 0)
    losses = torch.full((2,), -1.0, device="cuda")
    tr.step(torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda(), 1.0, 0.3, 2.0, losses)
    torch.cuda.synchronize()
    got = tr.get_weights()
    want, lp, ls = train.sgd_step(w, x, labels, Y, 1.0, 0.3, 2.0, arch)
    grads = train.gradients(w, x, labels, Y, 0.3, 2.0, arch)
    assert set(got) == set(want)
    if selector == "softmax":
        for k in want:
            tol = G_RTOL * np.max(np.abs(grads[k])) + ULP * np.max(np.abs(w[k]))
            assert np.max(np.abs(got[k].astype(np.float64) - want[k])) <= tol, k
    else:
        _check_update(got, want, w, grads, 1.0, where=f"fc_mlp {C}x{S}->{H}->{K} {selector}")
    lg = losses.cpu().numpy()
    assert abs(lg[0] - lp) <= 1e-5 * max(1.0, abs(lp)) and abs(lg[1] - ls) <= 1e-5 * max(1.0, abs(ls)), (lg, lp, ls)
    tr.close()


@pytest.mark.parametrize("C,ih,iw,Co,k,s,K,n,selector", [
    (4, 9, 8, 5, 3, 2, 6, 20, "linear"), (16, 14, 14, 8, 3, 1, 10, 24, "linear"), (8, 12, 12, 8, 5, 2, 33, 40, "hidden"),
    (3, 6, 6, 2, 6, 1, 4, 9, "softmax"),
    # shapes that the kernels working on the maps themselves take (3 x 3 / 5 x 5 taps, up to 8 filters), one per
    # way of dealing positions, channels and samples out: a partial channel group; four waves per map;
    # two waves per map; a ResNet stage-1 map; several samples per wave, per pass and a ragged last sample split
    (6, 30, 30, 8, 5, 2, 7, 10, "linear"), (5, 26, 24, 7, 3, 1, 5, 6, "linear"), (4, 40, 40, 8, 3, 2, 6, 7, "softmax"),
    (3, 56, 56, 8, 5, 2, 10, 5, "linear"), (8, 7, 7, 8, 3, 1, 6, 70, "linear"), (9, 5, 5, 3, 3, 1, 4, 133, "hidden"),
    (8, 9, 9, 12, 3, 1, 5, 12, "linear"),        # more than 8 filters: the product over gathered windows
])
def test_conv_predictor_step(C, ih, iw, Co, k, s, K, n, selector):
    """Conv(k,s): weight gradients of the filters, on the maps themselves or through the product over gathered
    windows; the caller's [filter][position] order of the hidden values survives the trainer's internal order."""
    rng = np.random.default_rng(C * ih + Co * k + s)
    oh, ow = (ih - k) // s + 1, (iw - k) // s + 1
    F = Co * oh * ow
    w = {"W1": rng.standard_normal((Co, C, k, k)) * np.sqrt(2.0 / (C * k * k)), "b1": rng.standard_normal(Co) * 0.1,
         "W2": rng.standard_normal((K, F)) * np.sqrt(2.0 / F), "b2": rng.standard_normal(K) * 0.1}
    if selector == "linear":
        w.update({"ws": rng.standard_normal(F + K) * 0.3, "bs": -0.1})
    elif selector == "hidden":
        w.update({"Ws": rng.standard_normal((6, F + K)) * 0.3, "cs": rng.standard_normal(6) * 0.1,
                  "vs": rng.standard_normal(6) * 0.5, "bs": -0.1})
    w = _w32(w)
    x = (rng.standard_normal((n, C, ih, iw)) + 0.2).astype(np.float32)
    labels = rng.integers(0, K, n).astype(np.int32)
    Y = _simplex(rng, n, K)
    arch = {"stride": s}
    f = train.forward(w, x, arch)
    z = np.sort(f["z"], axis=1)
    assert (z[:, -1] - z[:, -2]).min() > 1e-5 and np.abs(f["a"][np.abs(f["a"]) > 0]).min() > 1e-6
    tr = g.Trainer(C, Co, K, w, max_rows=n + 2, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s), selector=selector,
                   sel_hidden=6 if selector == "hidden" else 0)
    losses = torch.full((2,), -1.0, device="cuda")
    tr.step(torch.from_numpy(x.reshape(n, -1)).cuda(), torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda(),
            1.0, 0.4, 3.0, losses)
    torch.cuda.synchronize()
    got = tr.get_weights()
    want, lp, ls = train.sgd_step(w, x, labels, Y, 1.0, 0.4, 3.0, arch)
    grads = train.gradients(w, x, labels, Y, 0.4, 3.0, arch)
    assert set(got) == set(want) and got["W1"].shape == (Co, C, k, k)
    if selector == "softmax":
        for kk in want:
            tol = G_RTOL * np.max(np.abs(grads[kk])) + ULP * np.max(np.abs(w[kk]))
            assert np.max(np.abs(got[kk].astype(np.float64) - want[kk])) <= tol, kk
    else:
        _check_update(got, want, w, grads, 1.0, where=f"conv {C}x{ih}x{iw} k{k}s{s} {selector}")
    lg = losses.cpu().numpy()
    assert abs(lg[0] - lp) <= 1e-5 * max(1.0, abs(lp)) and abs(lg[1] - ls) <= 1e-5 * max(1.0, abs(ls)), (lg, lp, ls)
    tr.close()


@pytest.mark.parametrize("predictor", ["fc_mlp", "conv_fc"])
def test_retrain_then_serve_the_papers_gpu_predictors(predictor):
    """Five steps at the paper's learning rate on an fp32 cache of each kind, then the weights go into the
    serving cache and its lookups match the oracle's under the oracle-trained weights."""
    rng = np.random.default_rng(5 if predictor == "fc_mlp" else 6)
    n, C, ih, iw, K = 60, 8, 10, 10, 12
    S = ih * iw
    if predictor == "fc_mlp":
        H, kw, arch = 48, {}, {"sel_input": "hidden"}
        w = {"W1": rng.standard_normal((H, C * S)) * np.sqrt(2.0 / (C * S)), "b1": np.zeros(H),
             "W2": rng.standard_normal((K, H)) * np.sqrt(2.0 / H), "b2": np.zeros(K), "ws": rng.standard_normal(H + K) * 0.3, "bs": 0.0}
        d = oracle.CacheDef(C=C, S=S, H=H, K=K, predictor="fc_mlp", threshold=0.5)
    else:
        H, kw, arch = 8, dict(in_hw=(ih, iw), conv_ks=(3, 1)), {"stride": 1}
        F = H * 8 * 8
        w = {"W1": rng.standard_normal((H, C, 3, 3)) * np.sqrt(2.0 / (C * 9)), "b1": np.zeros(H),
             "W2": rng.standard_normal((K, F)) * np.sqrt(2.0 / F), "b2": np.zeros(K), "ws": rng.standard_normal(F + K) * 0.1, "bs": 0.0}
        d = oracle.CacheDef(C=C, S=S, H=H, K=K, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(3, 1), threshold=0.5)
    w = _w32(w)
    x = np.maximum(rng.standard_normal((n, C, ih, iw)) + 0.3, 0).astype(np.float32)
    labels = rng.integers(0, K, n).astype(np.int32)
    Y = _simplex(rng, n, K)
    x_or = x if predictor == "conv_fc" else x.reshape(n, -1)
    tr = g.Trainer(C, H, K, w, max_rows=n, predictor=predictor, S=S, **kw)
    xd, lab_d, Y_d = torch.from_numpy(x.reshape(n, -1)).cuda(), torch.from_numpy(labels).cuda(), torch.from_numpy(Y).cuda()
    cur = w
    lp0 = None
    for e in range(5):
        tr.step(xd, lab_d, Y_d, 0.002, 0.5, 3.0)
        cur, lp, ls = train.sgd_step(cur, x_or, labels, Y, 0.002, 0.5, 3.0, arch)
        lp0 = lp if lp0 is None else lp0
    torch.cuda.synchronize()
    got = tr.get_weights()
    assert lp < lp0
    for k in ("W1", "b1", "W2", "b2", "ws"):
        assert np.max(np.abs(got[k].astype(np.float64) - cur[k])) <= 1e-5 * max(1.0, np.max(np.abs(cur[k]))), k
    cache = g.Cache(C, S, H, K, "f32", "ncs", 0.5, n, got, predictor=predictor, **kw)
    w_or = {k: (np.asarray(v, np.float32) if k != "bs" else float(np.float32(v))) for k, v in cur.items()}
    want = oracle.lookup(d, w_or, x.reshape(n, C, S))
    pc = torch.empty(n, dtype=torch.int32, device="cuda")
    conf = torch.empty(n, device="cuda")
    hit = torch.empty(n, dtype=torch.uint8, device="cuda")
    logits = torch.empty((n, K), device="cuda")
    cache.lookup(torch.from_numpy(x.reshape(n, C, S)).cuda(), None, n, None, pc, conf, hit, logits)
    torch.cuda.synchronize()
    assert np.max(np.abs(logits.cpu().numpy() - want["logits"])) <= 1e-4
    assert np.max(np.abs(conf.cpu().numpy() - want["confidence"])) <= 1e-4
    zs = np.sort(want["logits"].astype(np.float64), axis=1)
    clear = (zs[:, -1] - zs[:, -2]) > 1e-3
    assert np.array_equal(pc.cpu().numpy()[clear], want["pred_class"][clear])
    tr.close(); cache.close()
