"""Pins for the paper's FC(h) predictor in the oracle (Section 3, table of predictor
architectures: Input(flattened) -FC-> Hidden Layer(h) -FC-> Output, ReLU)."""
import math

import numpy as np
import torch

from oracle import CacheDef


def _d(C, S, H, K, **kw):
    return CacheDef(C=C, S=S, H=H, K=K, predictor="fc_mlp", **kw)


def test_fc_mlp_hand_case(oracle):
    """D = C*S = 4 inputs [1,2,3,4] (C=2,S=2), H=2, K=2.
    W1 = [[1,0,-1,0],[0.5,0.5,0.5,0.5]], b1=[0,-10] -> h = (max(0,1-3), max(0,5-10)) = (0,0)?  use b1=[3,-4]:
    h = (max(0,1-3+3), max(0,5-4)) = (1,1).  W2=[[2,1],[1,1]], b2=[ln3-1,0] -> z=(2+ln3, 2), q=(3/4,1/4).
    selector over [h ; q]: ws=[1,-1,4,8] -> 1-1+3+2 = 5, bs = ln3-5 -> u = ln3, conf = 3/4."""
    ln3 = math.log(3.0)
    x = np.array([[[1, 2], [3, 4]]], np.float32)
    w = {"W1": np.array([[1, 0, -1, 0], [0.5, 0.5, 0.5, 0.5]], np.float32), "b1": np.array([3, -4], np.float32),
         "W2": np.array([[2, 1], [1, 1]], np.float32), "b2": np.array([ln3 - 1, 0], np.float32),
         "ws": np.array([1, -1, 4, 8], np.float32), "bs": ln3 - 5}
    out = oracle.lookup(_d(2, 2, 2, 2, threshold=0.7), w, x)
    assert out["pooled"].tolist() == [[1.0, 1.0]]          # the hidden layer is reported as the features
    assert abs(out["logits"][0, 0] - (2 + ln3)) < 1e-6 and abs(out["logits"][0, 1] - 2) < 1e-6
    assert abs(out["probs"][0, 0] - 0.75) < 1e-7 and out["pred_class"][0] == 0
    assert abs(out["score"][0] - ln3) < 1e-6 and abs(float(out["confidence"][0]) - 0.75) < 1e-6
    assert out["hit"][0] == 1
    # flatten order is storage order: W1 column e multiplies element e of the row as stored
    w2 = dict(w, W1=np.array([[0, 0, 0, 1], [0, 1, 0, 0]], np.float32), b1=np.zeros(2, np.float32))
    assert oracle.lookup(_d(2, 2, 2, 2), w2, x)["pooled"].tolist() == [[4.0, 2.0]]
    xt = np.ascontiguousarray(x.transpose(0, 2, 1))        # [n,S,C] storage: flattened (s,c) = [1,3,2,4]
    assert oracle.lookup(_d(2, 2, 2, 2, layout="nsc"), w2, xt)["pooled"].tolist() == [[4.0, 3.0]]


def test_fc_mlp_against_library_ops(oracle):
    g = np.random.default_rng(3)
    n, C, S, H, K = 4, 6, 8, 10, 7
    D = C * S
    x = g.standard_normal((n, C, S)).astype(np.float32)
    w = {"W1": (g.standard_normal((H, D)) * 0.2).astype(np.float32), "b1": (g.standard_normal(H) * 0.1).astype(np.float32),
         "W2": (g.standard_normal((K, H)) * 0.3).astype(np.float32), "b2": (g.standard_normal(K) * 0.1).astype(np.float32),
         "ws": (g.standard_normal(H + K) * 0.5).astype(np.float32), "bs": 0.1}
    out = oracle.lookup(_d(C, S, H, K, threshold=0.5), w, x)
    xf = torch.from_numpy(x).double().reshape(n, D)
    h = torch.relu(xf @ torch.from_numpy(w["W1"]).double().T + torch.from_numpy(w["b1"]).double()).float().double()
    z = h @ torch.from_numpy(w["W2"]).double().T + torch.from_numpy(w["b2"]).double()
    q = torch.softmax(z, dim=1)
    u = torch.cat([h, q], dim=1) @ torch.from_numpy(w["ws"]).double() + float(np.float32(0.1))
    assert np.allclose(out["pooled"], h.numpy(), atol=1e-6)
    assert np.allclose(out["logits"], z.numpy(), atol=1e-5)
    assert np.allclose(out["score"], u.numpy(), atol=1e-5)
    # bf16 operand arithmetic: x is bf16 data, W1/W2 and the hidden operand are rounded to bf16
    xb = torch.from_numpy(x).bfloat16()
    bits = xb.view(torch.int16).numpy().view(np.uint16)
    ob = oracle.lookup(_d(C, S, H, K, dtype="bf16", round_operands=True), w, bits)
    hb = torch.relu(xb.double().reshape(n, D) @ torch.from_numpy(w["W1"]).bfloat16().double().T
                    + torch.from_numpy(w["b1"]).double()).float()
    zb = hb.bfloat16().double() @ torch.from_numpy(w["W2"]).bfloat16().double().T + torch.from_numpy(w["b2"]).double()
    assert np.allclose(ob["pooled"], hb.numpy(), atol=1e-6)
    assert np.allclose(ob["logits"], zb.numpy(), atol=1e-5)
