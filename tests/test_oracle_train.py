"""Pins for the retraining-step oracle (Section 3, "Training Learned Caches"; Section 5,
"Retraining Learned Caches"): its gradients against finite differences of its own loss and against
an automatic-differentiation library, closed forms, and the direction of a step."""
import numpy as np
import torch

from oracle import train


def _case(seed=0, n=9, C=5, H=4, K=3):
    rng = np.random.default_rng(seed)
    w = {"W1": rng.standard_normal((H, C)) * 0.7, "b1": rng.standard_normal(H) * 0.2,
         "W2": rng.standard_normal((K, H)) * 0.7, "b2": rng.standard_normal(K) * 0.2,
         "ws": rng.standard_normal(C + K) * 0.5, "bs": 0.3}
    pooled = rng.standard_normal((n, C))
    labels = rng.integers(0, K, n)
    Y = rng.random((n, K)) + 0.05
    Y /= Y.sum(axis=1, keepdims=True)
    return w, pooled, labels, Y


def test_gradients_match_finite_differences_of_the_losses():
    w, pooled, labels, Y = _case()
    alpha, lam = 0.3, 2.5
    g = train.gradients(w, pooled, labels, Y, alpha, lam)
    eps = 1e-6
    for key, which in (("W1", 0), ("b1", 0), ("W2", 0), ("b2", 0), ("ws", 1)):
        flat = np.asarray(w[key], np.float64)
        for idx in list(np.ndindex(flat.shape))[:: max(1, flat.size // 7)]:
            wp = {k: np.array(v, np.float64) if k != "bs" else v for k, v in w.items()}
            wm = {k: np.array(v, np.float64) if k != "bs" else v for k, v in w.items()}
            wp[key][idx] += eps
            wm[key][idx] -= eps
            num = (train.losses(wp, pooled, labels, Y, alpha, lam)[which] -
                   train.losses(wm, pooled, labels, Y, alpha, lam)[which]) / (2 * eps)
            assert abs(num - g[key][idx]) < 1e-7, (key, idx, num, g[key][idx])
    num = (train.losses({**w, "bs": w["bs"] + eps}, pooled, labels, Y, alpha, lam)[1] -
           train.losses({**w, "bs": w["bs"] - eps}, pooled, labels, Y, alpha, lam)[1]) / (2 * eps)
    assert abs(num - g["bs"]) < 1e-7
    # the selector loss depends on W2 through q, yet the step's W2 gradient is the predictor loss's alone
    bump = np.array(w["W2"], np.float64)
    bump[0, 0] += 1e-3
    assert train.losses({**w, "W2": bump}, pooled, labels, Y, alpha, lam)[1] != \
        train.losses(w, pooled, labels, Y, alpha, lam)[1]


def test_against_automatic_differentiation():
    w, pooled, labels, Y = _case(seed=3, n=12, C=6, H=5, K=4)
    alpha, lam = 0.5, 3.0
    tw = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for k, v in w.items() if k != "bs"}
    bs = torch.tensor(float(w["bs"]), dtype=torch.float64, requires_grad=True)
    p = torch.tensor(pooled)
    h = torch.relu(p @ tw["W1"].T + tw["b1"])
    z = h @ tw["W2"].T + tw["b2"]
    logq = torch.log_softmax(z, dim=1)
    t = torch.tensor(train.targets(labels, Y, alpha))
    Lp = -(t * logq).sum() / len(labels)
    q = torch.softmax(z, dim=1).detach()                       # the selector sees the outputs as data
    u = torch.cat([p, q], dim=1) @ tw["ws"] + bs
    G = torch.tensor((z.detach().numpy().argmax(1) == Y.argmax(1)).astype(np.float64))
    Ls = -(G * torch.nn.functional.logsigmoid(u) + lam * (1 - G) * torch.nn.functional.logsigmoid(-u)).sum() / len(labels)
    (Lp + Ls).backward()
    g = train.gradients(w, pooled, labels, Y, alpha, lam)
    for k in ("W1", "b1", "W2", "b2", "ws"):
        assert np.max(np.abs(tw[k].grad.numpy() - g[k])) < 1e-12, k
    assert abs(bs.grad.item() - g["bs"]) < 1e-12
    lp, ls = train.losses(w, pooled, labels, Y, alpha, lam)
    assert abs(lp - Lp.item()) < 1e-12 and abs(ls - Ls.item()) < 1e-12


def test_closed_forms():
    w, pooled, labels, Y = _case(seed=5)
    n, K = Y.shape
    f = train.forward(w, pooled)
    # alpha = 0: plain cross-entropy on the labels, dz = (q - onehot) / n; db2 is its column sum
    g = train.gradients(w, pooled, labels, Y, 0.0, 1.0)
    one = np.eye(K)[labels]
    assert np.allclose(g["b2"], ((f["q"] - one) / n).sum(0), atol=1e-15)
    assert abs(g["b2"].sum()) < 1e-15                          # targets and probabilities both sum to one
    # alpha = 1 and a teacher equal to the predictor's own distribution: the predictor is at a stationary point
    g = train.gradients(w, pooled, labels, f["q"], 1.0, 1.0)
    assert max(np.max(np.abs(g[k])) for k in ("W1", "b1", "W2", "b2")) < 1e-15
    # fp_weight = 1: ordinary logistic regression on G; a larger weight scales exactly the G = 0 rows
    G = (f["z"].argmax(1) == Y.argmax(1)).astype(float)
    g1 = train.gradients(w, pooled, labels, Y, 0.3, 1.0)
    g4 = train.gradients(w, pooled, labels, Y, 0.3, 4.0)
    assert abs(g1["bs"] - ((f["c"] - G) / n).sum()) < 1e-15
    assert abs((g4["bs"] - g1["bs"]) - 3.0 * (((1 - G) * f["c"]) / n).sum()) < 1e-15
    assert 0 < G.sum() < n


def test_a_step_goes_downhill_and_zero_rate_is_the_identity():
    w, pooled, labels, Y = _case(seed=8, n=40, C=8, H=6, K=5)
    new, lp, ls = train.sgd_step(w, pooled, labels, Y, 0.0, 0.3, 2.0)
    assert all(np.array_equal(new[k], np.asarray(w[k], np.float64)) for k in ("W1", "b1", "W2", "b2", "ws"))
    cur = w
    for _ in range(5):                                          # the paper retrains for 5 epochs
        cur, lp1, ls1 = train.sgd_step(cur, pooled, labels, Y, 0.05, 0.3, 2.0)
    lp2 = train.losses(cur, pooled, labels, Y, 0.3, 2.0)[0]
    assert lp2 < lp and lp1 < lp


def _case_hidden(seed=0, n=9, C=5, H=4, K=3, Hs=6):
    w, pooled, labels, Y = _case(seed, n, C, H, K)
    rng = np.random.default_rng(seed + 100)
    del w["ws"]
    w.update({"Ws": rng.standard_normal((Hs, C + K)) * 0.6, "cs": rng.standard_normal(Hs) * 0.3,
              "vs": rng.standard_normal(Hs) * 0.8})
    return w, pooled, labels, Y


def test_hidden_layer_selector_gradients():
    """Finite differences of the oracle's own loss, and autograd on an independently written one."""
    w, pooled, labels, Y = _case_hidden(seed=2, n=11, C=6, H=5, K=4, Hs=7)
    alpha, lam = 0.4, 2.0
    g = train.gradients(w, pooled, labels, Y, alpha, lam)
    assert set(g) == {"W1", "b1", "W2", "b2", "Ws", "cs", "vs", "bs"}
    eps = 1e-6
    for key in ("Ws", "cs", "vs"):
        flat = np.asarray(w[key], np.float64)
        for idx in list(np.ndindex(flat.shape))[:: max(1, flat.size // 9)]:
            wp = {**w, key: flat.copy()}
            wm = {**w, key: flat.copy()}
            wp[key][idx] += eps
            wm[key][idx] -= eps
            num = (train.losses(wp, pooled, labels, Y, alpha, lam)[1] -
                   train.losses(wm, pooled, labels, Y, alpha, lam)[1]) / (2 * eps)
            assert abs(num - g[key][idx]) < 1e-7, (key, idx, num, g[key][idx])
    tw = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for k, v in w.items() if k != "bs"}
    bs = torch.tensor(float(w["bs"]), dtype=torch.float64, requires_grad=True)
    p = torch.tensor(pooled)
    z = torch.relu(p @ tw["W1"].T + tw["b1"]) @ tw["W2"].T + tw["b2"]
    q = torch.softmax(z, dim=1).detach()
    gh = torch.relu(torch.cat([p, q], dim=1) @ tw["Ws"].T + tw["cs"])
    u = gh @ tw["vs"] + bs
    G = torch.tensor((z.detach().numpy().argmax(1) == Y.argmax(1)).astype(np.float64))
    Ls = -(G * torch.nn.functional.logsigmoid(u) + lam * (1 - G) * torch.nn.functional.logsigmoid(-u)).sum() / len(labels)
    Ls.backward()
    for k in ("Ws", "cs", "vs"):
        assert np.max(np.abs(tw[k].grad.numpy() - g[k])) < 1e-12, k
    assert abs(bs.grad.item() - g["bs"]) < 1e-12
    assert tw["W1"].grad is None or float(tw["W1"].grad.abs().max()) == 0.0     # nothing reaches the predictor
    assert abs(train.losses(w, pooled, labels, Y, alpha, lam)[1] - Ls.item()) < 1e-12


def test_hidden_layer_selector_limits():
    """One always-active unit with vs = 1 and cs = 0 is the linear selector; a unit that the ReLU clamps
    for every sample gets no gradient."""
    w, pooled, labels, Y = _case(seed=4)
    lin = train.gradients(w, pooled, labels, Y, 0.3, 2.0)
    f = train.forward(w, pooled)
    shift = 1.0 - f["x"] @ w["ws"]                       # keep the single unit positive for every sample
    big = float(shift.max()) + 1.0
    wh = {k: v for k, v in w.items() if k != "ws"}
    wh.update({"Ws": np.asarray(w["ws"])[None, :], "cs": np.array([big]), "vs": np.array([1.0]), "bs": w["bs"] - big})
    fh = train.forward(wh, pooled)
    assert np.allclose(fh["u"], f["u"], atol=1e-12)
    gh = train.gradients(wh, pooled, labels, Y, 0.3, 2.0)
    assert np.allclose(gh["Ws"][0], lin["ws"], atol=1e-12) and abs(gh["cs"][0] - lin["bs"]) < 1e-12
    wd = {**wh, "Ws": np.vstack([wh["Ws"], -wh["Ws"]]), "cs": np.array([big, -big - 50.0]), "vs": np.array([1.0, 0.7])}
    gd = train.gradients(wd, pooled, labels, Y, 0.3, 2.0)
    assert np.all(gd["Ws"][1] == 0.0) and gd["cs"][1] == 0.0 and gd["vs"][1] == 0.0


def test_pool_fc_predictor_is_softmax_regression():
    """Without a hidden layer the predictor is multinomial logistic regression on the features: the
    gradient has the closed form (q - t)^T f / n, and it equals the two-layer network whose first layer is
    the identity on non-negative features."""
    w, pooled, labels, Y = _case(seed=6, n=10, C=5, H=5, K=4)
    feats = np.abs(pooled)                                     # ReLU'd window means are non-negative
    wp = {"W2": np.random.default_rng(1).standard_normal((4, 5)) * 0.5, "b2": w["b2"], "ws": w["ws"], "bs": w["bs"]}
    g = train.gradients(wp, feats, labels, Y, 0.3, 2.0)
    assert set(g) == {"W2", "b2", "ws", "bs"}
    f = train.forward(wp, feats)
    t = train.targets(labels, Y, 0.3)
    assert np.allclose(g["W2"], (f["q"] - t).T @ feats / len(labels), atol=1e-15)
    two = {**wp, "W1": np.eye(5), "b1": np.zeros(5)}
    g2 = train.gradients(two, feats, labels, Y, 0.3, 2.0)
    for k in ("W2", "b2", "ws"):
        assert np.allclose(g[k], g2[k], atol=1e-15), k
    assert train.losses(wp, feats, labels, Y, 0.3, 2.0) == train.losses(two, feats, labels, Y, 0.3, 2.0)
    eps = 1e-6
    bump = wp["W2"].copy(); bump[1, 2] += eps
    low = wp["W2"].copy(); low[1, 2] -= eps
    num = (train.losses({**wp, "W2": bump}, feats, labels, Y, 0.3, 2.0)[0] -
           train.losses({**wp, "W2": low}, feats, labels, Y, 0.3, 2.0)[0]) / (2 * eps)
    assert abs(num - g["W2"][1, 2]) < 1e-7


def _fd_check(w, x, labels, Y, alpha, lam, arch, keys, which):
    g = train.gradients(w, x, labels, Y, alpha, lam, arch)
    eps = 1e-6
    for key in keys:
        flat = np.asarray(w[key], np.float64)
        for idx in list(np.ndindex(flat.shape))[:: max(1, flat.size // 9)]:
            wp = {**w, key: flat.copy()}
            wm = {**w, key: flat.copy()}
            wp[key][idx] += eps
            wm[key][idx] -= eps
            num = (train.losses(wp, x, labels, Y, alpha, lam, arch)[which] -
                   train.losses(wm, x, labels, Y, alpha, lam, arch)[which]) / (2 * eps)
            assert abs(num - g[key][idx]) < 1e-7, (key, idx, num, g[key][idx])
    return g


def test_fc_predictor_whose_selector_reads_the_hidden_layer():
    """FC(h): the same two-layer network on the flattened row; the selector reads [h ; q] and treats both as
    data.  Finite differences, autograd on an independently written loss, and the predictor's gradients must
    not depend on which features the selector reads."""
    rng = np.random.default_rng(21)
    n, D, H, K = 10, 12, 5, 4
    w = {"W1": rng.standard_normal((H, D)) * 0.5, "b1": rng.standard_normal(H) * 0.2, "W2": rng.standard_normal((K, H)) * 0.7,
         "b2": rng.standard_normal(K) * 0.2, "ws": rng.standard_normal(H + K) * 0.5, "bs": -0.2}
    x = np.maximum(rng.standard_normal((n, D)), 0)
    labels = rng.integers(0, K, n)
    Y = rng.random((n, K)) + 0.05
    Y /= Y.sum(axis=1, keepdims=True)
    arch = {"sel_input": "hidden"}
    g = _fd_check(w, x, labels, Y, 0.4, 2.0, arch, ("W1", "b1", "W2", "b2"), 0)
    _fd_check(w, x, labels, Y, 0.4, 2.0, arch, ("ws",), 1)
    tw = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for k, v in w.items() if k != "bs"}
    bs = torch.tensor(float(w["bs"]), dtype=torch.float64, requires_grad=True)
    h = torch.relu(torch.tensor(x) @ tw["W1"].T + tw["b1"])
    z = h @ tw["W2"].T + tw["b2"]
    Lp = -(torch.tensor(train.targets(labels, Y, 0.4)) * torch.log_softmax(z, dim=1)).sum() / n
    u = torch.cat([h.detach(), torch.softmax(z, dim=1).detach()], dim=1) @ tw["ws"] + bs
    G = torch.tensor((z.detach().numpy().argmax(1) == Y.argmax(1)).astype(np.float64))
    Ls = -(G * torch.nn.functional.logsigmoid(u) + 2.0 * (1 - G) * torch.nn.functional.logsigmoid(-u)).sum() / n
    (Lp + Ls).backward()
    for k in ("W1", "b1", "W2", "b2", "ws"):
        assert np.max(np.abs(tw[k].grad.numpy() - g[k])) < 1e-12, k
    assert abs(bs.grad.item() - g["bs"]) < 1e-12
    # the predictor's part equals that of a network whose selector reads the input instead
    wi = {**w, "ws": rng.standard_normal(D + K)}
    gi = train.gradients(wi, x, labels, Y, 0.4, 2.0, {"sel_input": "input"})
    for k in ("W1", "b1", "W2", "b2"):
        assert np.array_equal(g[k], gi[k]), k
    assert g["ws"].shape == (H + K,) and gi["ws"].shape == (D + K,)


def test_conv_predictor_gradients():
    """Conv(k,s): finite differences, autograd through the library's convolution, and the full-size filter,
    which must give the FC(h) gradients on the flattened map."""
    rng = np.random.default_rng(22)
    n, C, ih, iw, Co, k, s, K = 6, 3, 7, 6, 4, 3, 2, 5
    oh, ow = (ih - k) // s + 1, (iw - k) // s + 1
    F = Co * oh * ow
    w = {"W1": rng.standard_normal((Co, C, k, k)) * 0.4, "b1": rng.standard_normal(Co) * 0.2,
         "W2": rng.standard_normal((K, F)) * 0.4, "b2": rng.standard_normal(K) * 0.2,
         "ws": rng.standard_normal(F + K) * 0.4, "bs": 0.1}
    x = rng.standard_normal((n, C, ih, iw))
    labels = rng.integers(0, K, n)
    Y = rng.random((n, K)) + 0.05
    Y /= Y.sum(axis=1, keepdims=True)
    arch = {"stride": s}
    f = train.forward(w, x, arch)
    assert f["h"].shape == (n, F)
    ref = torch.relu(torch.nn.functional.conv2d(torch.tensor(x), torch.tensor(w["W1"]), torch.tensor(w["b1"]), stride=s))
    assert np.allclose(f["h"], ref.reshape(n, -1).numpy(), atol=1e-12)          # [filter][oy][ox] order
    g = _fd_check(w, x, labels, Y, 0.3, 2.5, arch, ("W1", "b1", "W2", "b2"), 0)
    _fd_check(w, x, labels, Y, 0.3, 2.5, arch, ("ws",), 1)
    tw = {kk: torch.tensor(np.asarray(v, np.float64), requires_grad=True) for kk, v in w.items() if kk != "bs"}
    bs = torch.tensor(float(w["bs"]), dtype=torch.float64, requires_grad=True)
    h = torch.relu(torch.nn.functional.conv2d(torch.tensor(x), tw["W1"], tw["b1"], stride=s)).reshape(n, -1)
    z = h @ tw["W2"].T + tw["b2"]
    Lp = -(torch.tensor(train.targets(labels, Y, 0.3)) * torch.log_softmax(z, dim=1)).sum() / n
    u = torch.cat([h.detach(), torch.softmax(z, dim=1).detach()], dim=1) @ tw["ws"] + bs
    G = torch.tensor((z.detach().numpy().argmax(1) == Y.argmax(1)).astype(np.float64))
    Ls = -(G * torch.nn.functional.logsigmoid(u) + 2.5 * (1 - G) * torch.nn.functional.logsigmoid(-u)).sum() / n
    (Lp + Ls).backward()
    for kk in ("W1", "b1", "W2", "b2", "ws"):
        assert np.max(np.abs(tw[kk].grad.numpy() - g[kk])) < 1e-12, kk
    lp, ls = train.losses(w, x, labels, Y, 0.3, 2.5, arch)
    assert abs(lp - Lp.item()) < 1e-12 and abs(ls - Ls.item()) < 1e-12
    # a filter as large as the (square) map: one output position per filter = FC over the flattened map
    xs = rng.standard_normal((n, C, 4, 4))
    wf = {"W1": rng.standard_normal((Co, C, 4, 4)) * 0.3, "b1": w["b1"], "W2": rng.standard_normal((K, Co)) * 0.5,
          "b2": w["b2"], "ws": rng.standard_normal(Co + K) * 0.4, "bs": 0.1}
    gc = train.gradients(wf, xs, labels, Y, 0.3, 2.5, {"stride": 1})
    gf = train.gradients({**wf, "W1": wf["W1"].reshape(Co, -1)}, xs.reshape(n, -1), labels, Y, 0.3, 2.5, {"sel_input": "hidden"})
    assert np.allclose(gc["W1"].reshape(Co, -1), gf["W1"], atol=1e-14)
    for kk in ("b1", "W2", "b2", "ws"):
        assert np.allclose(gc[kk], gf[kk], atol=1e-14), kk


def test_softmax_threshold_mode_trains_the_predictor_alone():
    """No selector network: the predictor's gradients equal those of the same network with a selector, the
    selector loss is zero and no selector gradient exists."""
    w, pooled, labels, Y = _case(seed=9)
    g = train.gradients(w, pooled, labels, Y, 0.3, 2.0)
    bare = {k: v for k, v in w.items() if k not in ("ws", "bs")}
    gb = train.gradients(bare, pooled, labels, Y, 0.3, 2.0)
    assert set(gb) == {"W1", "b1", "W2", "b2"}
    for k in gb:
        assert np.array_equal(gb[k], g[k]), k
    assert train.losses(bare, pooled, labels, Y, 0.3, 2.0) == (train.losses(w, pooled, labels, Y, 0.3, 2.0)[0], 0.0)
    new, lp, ls = train.sgd_step(bare, pooled, labels, Y, 0.1, 0.3, 2.0)
    assert set(new) == {"W1", "b1", "W2", "b2"} and ls == 0.0
