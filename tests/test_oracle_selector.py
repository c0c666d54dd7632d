"""Pins for the selector (Section 3, "Selector Network Design"; T = sigma_i(PR))
and for the whole lookup on a hand-computed case."""
import math

import numpy as np

from oracle import CacheDef

LN3 = math.log(3.0)


def _w(C, H, K, **kw):
    w = {"W1": np.zeros((H, C), np.float32), "b1": np.zeros(H, np.float32),
         "W2": np.zeros((K, H), np.float32), "b2": np.zeros(K, np.float32),
         "ws": np.zeros(C + K, np.float32), "bs": 0.0}
    for k, v in kw.items():
        w[k] = v if k == "bs" else np.asarray(v, np.float32)
    return w


def test_score_hand_case(oracle):
    d = CacheDef(C=2, S=1, H=1, K=2)
    w = _w(2, 1, 2, ws=[0.5, -1, 4, 8], bs=-4.5)
    # 0.5*2 - 1*1 + 4*0.75 + 8*0.25 - 4.5 = 1 - 1 + 3 + 2 - 4.5 = 0.5
    u = oracle.selector_score(d, w, np.array([2, 1], np.float32), np.array([0.75, 0.25]))
    assert u == 0.5
    # pooled part comes first in ws: swapping the halves changes the result
    w2 = _w(2, 1, 2, ws=[4, 8, 0.5, -1], bs=-4.5)
    assert oracle.selector_score(d, w2, np.array([2, 1], np.float32), np.array([0.75, 0.25])) == 8 + 8 + 0.375 - 0.25 - 4.5


def test_zero_selector_weights_and_threshold_edges(oracle):
    x = np.random.default_rng(0).standard_normal((5, 3, 4)).astype(np.float32)
    for tau, want in ((0.5, 0), (0.4999, 1), (0.0, 1), (1.0, 0)):
        d = CacheDef(C=3, S=4, H=2, K=3, threshold=tau)
        out = oracle.lookup(d, _w(3, 2, 3), x)
        assert np.all(out["confidence"] == np.float32(0.5))      # logistic(0)
        assert np.all(out["hit"] == want), tau                   # strictly above tau
    # confidence = logistic(bs) when ws = 0, monotone in bs
    prev = -1.0
    for bs in (-30.0, -2.0, 0.0, LN3, 40.0):
        d = CacheDef(C=3, S=4, H=2, K=3, threshold=1.0)
        out = oracle.lookup(d, _w(3, 2, 3, bs=bs), x)
        want = 1.0 / (1.0 + math.exp(-bs))
        assert abs(float(out["confidence"][0]) - want) < 1e-7
        assert float(out["confidence"][0]) >= prev
        prev = float(out["confidence"][0])
        assert np.all(out["hit"] == 0)      # tau = 1: never a hit, even when logistic saturates to 1.0f


def test_full_lookup_hand_case(oracle):
    """C=2, S=3, H=2, K=2, three rows; every intermediate worked by hand.

    row0: p=(2,1)  h=(max(0,2-1), max(0,1+2-5))=(1,0)  z=(2+ln3, 1+1)=(2+ln3, 2)
          q=(3/4,1/4) cls=0  u = bs + .5*2 - 1*1 + 4*.75 + 8*.25 = bs + 5
    row1: p=(3,-3) h=(6, max(0,1.5-6-5))=(6,0)        z=(12+ln3, 7)  z0-z1 = 5+ln3
          q1 = 1/(1+3e^5) cls=0 u = bs + 1.5 + 3 + 4 q0 + 8 q1 = bs + 8.5 + 4 q1
    row2: p=(0,3)  h=(max(0,-3), max(0,6-5))=(0,1)    z=(-7+ln3, 3+1)=(-7+ln3, 4)
          z1-z0 = 11-ln3, q0 = 1/(1+e^11/3) cls=1  u = bs - 3 + 4 q0 + 8 q1 = bs + 5 - 4 q0
    bs = ln3 - 5  =>  row0: u = ln3, confidence = 3/4.
    """
    x = np.array([[[1, 2, 3], [-1, 0, 4]],
                  [[3, 3, 3], [-3, -3, -3]],
                  [[0, 0, 0], [2, 3, 4]]], np.float32)
    w = _w(2, 2, 2, W1=[[1, -1], [0.5, 2]], b1=[0, -5], W2=[[2, -7], [1, 3]], b2=[LN3, 1],
           ws=[0.5, -1, 4, 8], bs=LN3 - 5.0)
    d = CacheDef(C=2, S=3, H=2, K=2, threshold=0.7)
    out = oracle.lookup(d, w, x)
    assert out["pooled"].tolist() == [[2, 1], [3, -3], [0, 3]]
    f32 = np.float32
    b20 = float(f32(LN3))             # the weights are fp32 inputs
    bs = float(f32(LN3 - 5.0))
    z = [[2 + b20, 2.0], [12 + b20, 7.0], [-7 + b20, 4.0]]
    assert np.array_equal(out["logits"], np.array(z, np.float64).astype(f32))
    assert out["pred_class"].tolist() == [0, 0, 1]
    q1_row1 = 1.0 / (1.0 + math.exp(5 + b20))
    q0_row2 = 1.0 / (1.0 + math.exp(11 - b20))
    assert abs(out["probs"][0, 0] - 0.75) < 1e-7 and abs(out["probs"][0, 1] - 0.25) < 1e-7
    assert abs(out["probs"][1, 1] - q1_row1) < 1e-15
    assert abs(out["probs"][2, 0] - q0_row2) < 1e-15
    q0_row0 = 1.0 / (1.0 + math.exp(-b20))
    u = [bs + 1 - 1 + 4 * q0_row0 + 8 * (1 - q0_row0),
         bs + 8.5 + 4 * q1_row1,
         bs + 5 - 4 * q0_row2]
    assert np.allclose(out["score"], u, rtol=0, atol=1e-13)
    assert abs(out["score"][0] - LN3) < 1e-6
    conf = [1 / (1 + math.exp(-v)) for v in u]
    assert np.allclose(out["confidence"], conf, rtol=0, atol=1e-7)
    assert abs(float(out["confidence"][0]) - 0.75) < 1e-6
    assert out["hit"].tolist() == [1, 1, 1]            # 0.75, ~0.99, ~0.75 all above 0.7
    # raise the threshold between row0/row2 (~0.75) and row1 (~0.99)
    d2 = CacheDef(C=2, S=3, H=2, K=2, threshold=0.9)
    assert oracle.lookup(d2, w, x)["hit"].tolist() == [0, 1, 0]
    # the same rows through a gather list and through the [n,S,C] layout
    out_g = oracle.lookup(d, w, x, row_index=np.array([2, 0], np.int32))
    assert np.array_equal(out_g["logits"], out["logits"][[2, 0]])
    assert out_g["pred_class"].tolist() == [1, 0]
    d3 = CacheDef(C=2, S=3, H=2, K=2, threshold=0.7, layout="nsc")
    out_t = oracle.lookup(d3, w, np.ascontiguousarray(x.transpose(0, 2, 1)))
    assert np.array_equal(out_t["logits"], out["logits"])
    assert np.array_equal(out_t["confidence"], out["confidence"])


def test_lookup_composes_the_steps_against_library_ops(oracle):
    """Whole lookup vs the same map assembled from library routines (third opinion)."""
    import torch
    g = np.random.default_rng(11)
    n, C, S, H, K = 6, 13, 9, 17, 23
    x = g.standard_normal((n, C, S)).astype(np.float32)
    w = _w(C, H, K, W1=g.standard_normal((H, C)) * 0.3, b1=g.standard_normal(H) * 0.1,
           W2=g.standard_normal((K, H)) * 0.3, b2=g.standard_normal(K) * 0.1,
           ws=g.standard_normal(C + K) * 0.5, bs=0.2)
    d = CacheDef(C=C, S=S, H=H, K=K, threshold=0.55)
    out = oracle.lookup(d, w, x)
    xt = torch.from_numpy(x).double()
    p = xt.mean(dim=2).float().double()
    h = torch.relu(torch.nn.functional.linear(p, torch.from_numpy(w["W1"]).double(), torch.from_numpy(w["b1"]).double()))
    z = torch.nn.functional.linear(h, torch.from_numpy(w["W2"]).double(), torch.from_numpy(w["b2"]).double())
    q = torch.softmax(z, dim=1)
    u = torch.cat([p, q], dim=1) @ torch.from_numpy(w["ws"]).double() + float(np.float32(0.2))
    conf = torch.sigmoid(u)
    assert np.allclose(out["logits"], z.numpy(), rtol=0, atol=1e-6)
    assert np.allclose(out["probs"], q.numpy(), rtol=0, atol=1e-12)
    assert np.array_equal(out["pred_class"], z.float().argmax(dim=1).numpy())
    assert np.allclose(out["score"], u.numpy(), rtol=0, atol=1e-12)
    assert np.allclose(out["confidence"], conf.numpy(), rtol=0, atol=1e-7)
    assert np.array_equal(out["hit"], (conf.float().numpy() > np.float32(0.55)).astype(np.uint8))


def test_softmax_threshold_mode(oracle):
    """No selector network: confidence is the top class probability (Appendix, design analysis:
    the baseline that thresholds the predictor's softmax scores)."""
    import torch
    g = np.random.default_rng(21)
    n, C, S, H, K = 7, 6, 4, 5, 9
    x = g.standard_normal((n, C, S)).astype(np.float32)
    w = _w(C, H, K, W1=g.standard_normal((H, C)), b1=g.standard_normal(H) * 0.1,
           W2=g.standard_normal((K, H)), b2=g.standard_normal(K) * 0.1,
           ws=g.standard_normal(C + K) * 5, bs=3.0)          # selector weights must be ignored
    d = CacheDef(C=C, S=S, H=H, K=K, threshold=0.5, selector="softmax")
    out = oracle.lookup(d, w, x)
    z = torch.from_numpy(out["logits"].astype(np.float64))
    assert np.allclose(out["confidence"], out["probs"].max(axis=1), rtol=0, atol=1e-7)
    assert np.allclose(out["confidence"], torch.softmax(z, dim=1).max(dim=1).values.numpy(), atol=1e-6)
    assert np.array_equal(out["hit"], (out["confidence"] > np.float32(0.5)).astype(np.uint8))
    assert np.array_equal(out["pred_class"], out["probs"].argmax(axis=1))
    # K = 2: top probability = logistic(|z0 - z1|); with |z0 - z1| = ln 3 it is exactly 3/4
    d2 = CacheDef(C=2, S=3, H=2, K=2, threshold=0.7, selector="softmax")
    w2 = _w(2, 2, 2, W1=[[1, -1], [0.5, 2]], b1=[0, -5], W2=[[2, -7], [1, 3]], b2=[LN3, 1], ws=[9, 9, 9, 9], bs=9)
    x2 = np.array([[[1, 2, 3], [-1, 0, 4]]], np.float32)
    o2 = oracle.lookup(d2, w2, x2)
    assert abs(float(o2["confidence"][0]) - 0.75) < 1e-6 and o2["hit"][0] == 1
    # hit set shrinks monotonically as the threshold rises; a uniform distribution gives 1/K
    hits = [int(oracle.lookup(CacheDef(C=C, S=S, H=H, K=K, threshold=t, selector="softmax"), w, x)["hit"].sum())
            for t in (0.0, 0.2, 0.5, 0.9, 1.0)]
    assert hits[0] == n and hits[-1] == 0 and all(a >= b for a, b in zip(hits, hits[1:]))
    w0 = _w(C, H, K)
    assert np.allclose(oracle.lookup(d, w0, x)["confidence"], 1.0 / K, atol=1e-7)


# ---- the selector with one hidden layer (Section 3, "Selector Network Design") ----

def test_hidden_selector_hand_case(oracle):
    """F = 2, K = 2, two hidden units; p = (1, 2), q = (3/4, 1/4).

    g0 = relu(0 + 1*1 + 0*2 + 4*.75 + 0*.25) = 4
    g1 = relu(-1 - 1*1 + 1*2 + 0*.75 + 4*.25) = 1
    u  = 0.5 + 2*4 - 1*1 = 7.5
    """
    d = CacheDef(C=2, S=1, H=1, K=2, selector="hidden", sel_hidden=2)
    w = _w(2, 1, 2, Ws=[[1, 0, 4, 0], [-1, 1, 0, 4]], cs=[0, -1], vs=[2, -1], bs=0.5)
    p, q = np.array([1, 2], np.float32), np.array([0.75, 0.25])
    assert oracle.selector_hidden_score(d, w, p, q) == 7.5
    # the ReLU clamps: push unit 1 below zero and it drops out (u = 0.5 + 8)
    w["cs"] = np.asarray([0, -3], np.float32)
    assert oracle.selector_hidden_score(d, w, p, q) == 8.5
    # features come first in a row of Ws, and rows are hidden units: probe both with an index pattern
    Ws = np.array([[10 * j + i for i in range(4)] for j in range(2)], np.float32)      # Ws[j,i] = 10j+i
    w = _w(2, 1, 2, Ws=Ws, cs=[0, 0], vs=[1, 100], bs=0.0)
    for i in range(4):                      # one-hot input i picks column i of both rows
        x = np.zeros(4)
        x[i] = 1.0
        got = oracle.selector_hidden_score(d, w, x[:2].astype(np.float32), x[2:])
        assert got == i + 100 * (10 + i)


def test_hidden_selector_against_library_ops_and_linear_limit(oracle):
    rng = np.random.default_rng(5)
    F, K, Hs = 7, 5, 6
    d = CacheDef(C=F, S=1, H=1, K=K, selector="hidden", sel_hidden=Hs)
    Ws = rng.standard_normal((Hs, F + K)).astype(np.float32)
    cs = rng.standard_normal(Hs).astype(np.float32)
    vs = rng.standard_normal(Hs).astype(np.float32)
    p = rng.standard_normal(F).astype(np.float32)
    q = rng.random(K)
    q /= q.sum()
    w = _w(F, 1, K, Ws=Ws, cs=cs, vs=vs, bs=0.25)
    x = np.concatenate([p.astype(np.float64), q])
    want = 0.25 + vs.astype(np.float64) @ np.maximum(Ws.astype(np.float64) @ x + cs, 0.0)
    assert abs(oracle.selector_hidden_score(d, w, p, q) - want) < 1e-12
    # one always-active unit with unit output weight is the single-layer selector
    ws = rng.standard_normal(F + K).astype(np.float32)
    d1 = CacheDef(C=F, S=1, H=1, K=K, selector="hidden", sel_hidden=1)
    w1 = _w(F, 1, K, Ws=ws[None, :], cs=[64.0], vs=[1.0], bs=-64.0 + 0.5)
    lin = oracle.selector_score(CacheDef(C=F, S=1, H=1, K=K), _w(F, 1, K, ws=ws, bs=0.5), p, q)
    assert abs(oracle.selector_hidden_score(d1, w1, p, q) - lin) < 1e-12


def test_hidden_selector_bf16_rounding_points(oracle):
    """bf16 cache arithmetic: first-layer weights, its operands and the hidden vector are rounded
    (nearest even); the second layer is not.  1 + 2^-8 is a tie and rounds to 1:
    Ws = 1+2^-8 -> 1, p = 3 -> g = 3, vs = 1+2^-8 stays: u = 3*(1+2^-8)."""
    d = CacheDef(C=1, S=1, H=1, K=1, selector="hidden", sel_hidden=1, round_operands=True)
    e = 2.0 ** -8
    w = _w(1, 1, 1, Ws=[[1 + e, 0]], cs=[0], vs=[1 + e], bs=0.0)
    assert oracle.selector_hidden_score(d, w, np.array([3], np.float32), np.array([1.0])) == 3 * (1 + e)
    d0 = CacheDef(C=1, S=1, H=1, K=1, selector="hidden", sel_hidden=1)
    assert oracle.selector_hidden_score(d0, w, np.array([3], np.float32), np.array([1.0])) == 3 * (1 + e) * (1 + e)
    # the hidden vector itself is rounded: g = 1 + 2^-8 + 2^-9 (exact sum of bf16 products) -> 1 + 2^-7
    w = _w(1, 1, 1, Ws=[[1, 0]], cs=[e / 2], vs=[1], bs=0.0)
    got = oracle.selector_hidden_score(d, w, np.array([1 + 2 * e], np.float32), np.array([1.0]))
    assert got == 1 + 2 * e          # 1 + 2^-7 + 2^-9 rounds down to 1 + 2^-7


def test_hidden_selector_in_lookup(oracle):
    """The full-lookup hand case (see test_full_lookup_hand_case), row 0, with a hidden-layer selector:
    p = (2, 1), q = (3/4, 1/4); g = relu(.5*2 - 1*1 + 4*.75 + 8*.25 - 4) = 1; u = ln3 * 1 -> conf 3/4."""
    d = CacheDef(C=2, S=3, H=2, K=2, threshold=0.7, selector="hidden", sel_hidden=1)
    x = np.array([[[1, 2, 3], [0, 1, 2]]], np.float32)
    w = _w(2, 2, 2, W1=[[1, -1], [1, 2]], b1=[0, -5], W2=[[2, 0], [1, 0]], b2=[LN3, 1],
           Ws=[[0.5, -1, 4, 8]], cs=[-4.0], vs=[LN3], bs=0.0)
    out = oracle.lookup(d, w, x)
    assert abs(float(out["confidence"][0]) - 0.75) < 1e-7 and out["hit"][0] == 1 and out["pred_class"][0] == 0
