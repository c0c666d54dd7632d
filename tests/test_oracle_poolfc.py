"""Pins for the paper's Pool(h) predictor in the oracle (Section 3, table of predictor
architectures: Input -Pool-> Hidden Layer(h) -FC-> Output, ReLU): adaptive average pool to
an out_h x out_w map, ReLU, one FC."""
import math

import numpy as np
import torch

from oracle import CacheDef


def _d(C, ih, iw, oh, ow, K=2, dtype="f32", **kw):
    return CacheDef(C=C, S=ih * iw, H=0, K=K, dtype=dtype, predictor="pool_fc", in_hw=(ih, iw), out_hw=(oh, ow), **kw)


def test_adaptive_pool_hand_cases(oracle):
    # one channel, 4x4 -> 2x2: plain 2x2 blocks
    x = np.arange(16, dtype=np.float32).reshape(1, 1, 16)
    f = oracle.pool(_d(1, 4, 4, 2, 2), x)
    assert f.tolist() == [[2.5, 4.5, 10.5, 12.5]]          # (0+1+4+5)/4, (2+3+6+7)/4, ...
    # 3x3 -> 2x2: windows [0,2) and [1,3) overlap on the middle row / column
    x = np.arange(9, dtype=np.float32).reshape(1, 1, 9)
    f = oracle.pool(_d(1, 3, 3, 2, 2), x)
    assert f.tolist() == [[2.0, 3.0, 5.0, 6.0]]            # (0+1+3+4)/4, (1+2+4+5)/4, (3+4+6+7)/4, (4+5+7+8)/4
    # negative means are clipped by the ReLU of the hidden layer
    x = -np.arange(16, dtype=np.float32).reshape(1, 1, 16)
    assert oracle.pool(_d(1, 4, 4, 2, 2), x).tolist() == [[0.0, 0.0, 0.0, 0.0]]
    # feature order is [channel][oy][ox]; non-square maps
    x = np.stack([np.arange(8, dtype=np.float32), 100 + np.arange(8, dtype=np.float32)]).reshape(1, 2, 8)
    f = oracle.pool(_d(2, 2, 4, 1, 2), x)                  # 2 rows x 4 cols -> 1 x 2
    assert f.tolist() == [[2.5, 4.5, 102.5, 104.5]]        # (0+1+4+5)/4, (2+3+6+7)/4


def test_adaptive_pool_limits(oracle):
    g = np.random.default_rng(0)
    x = np.abs(g.standard_normal((3, 5, 42))).astype(np.float32)
    # 1x1 output = global mean (values are non-negative, so the ReLU is the identity)
    glob = oracle.pool(CacheDef(C=5, S=42, H=1, K=1), x)
    assert np.array_equal(oracle.pool(_d(5, 6, 7, 1, 1), x), glob)
    # output map = input map: every window is one element
    assert np.array_equal(oracle.pool(_d(5, 6, 7, 6, 7), x).reshape(3, 5, 42), x)


def test_adaptive_pool_against_library(oracle):
    g = np.random.default_rng(1)
    for (C, ih, iw, oh, ow) in [(3, 7, 7, 2, 2), (2, 14, 14, 4, 4), (4, 5, 9, 3, 2), (2, 56, 56, 4, 4),
                                (1, 16, 16, 8, 8), (3, 10, 7, 10, 3)]:
        x = g.standard_normal((2, C, ih * iw)).astype(np.float32)
        want = torch.nn.functional.adaptive_avg_pool2d(torch.from_numpy(x).double().reshape(2, C, ih, iw), (oh, ow))
        want = torch.relu(want).reshape(2, -1).numpy()
        got = oracle.pool(_d(C, ih, iw, oh, ow), x)
        assert np.allclose(got, want, rtol=0, atol=1e-6), (C, ih, iw, oh, ow)
    t = torch.randn(2, 3, 49, generator=torch.Generator().manual_seed(2)).bfloat16()
    bits = t.view(torch.int16).numpy().view(np.uint16)
    want = torch.relu(torch.nn.functional.adaptive_avg_pool2d(t.double().reshape(2, 3, 7, 7), (2, 2))).reshape(2, -1)
    assert np.allclose(oracle.pool(_d(3, 7, 7, 2, 2, dtype="bf16"), bits), want.numpy(), atol=1e-6)


def test_pool_fc_lookup_hand_case(oracle):
    """C=1, 2x2 map pooled to 1x2 (F=2), K=2.  x = [[1,3],[5,7]] -> columns: (1+5)/2=3, (3+7)/2=5.
    z = W2 f + b2 = (1*3 - 1*5 + ln3 + 2, 0) with W2 = [[1,-1],[0,0]], b2 = [ln3+2, 0] -> z0 - z1 = ln 3,
    q = (3/4, 1/4), cls 0.  u = bs + .5*3 - .5*5 + 4*.75 + 8*.25 = bs + 4 ; bs = ln3 - 4 -> conf = 3/4."""
    ln3 = math.log(3.0)
    x = np.array([[[1, 3, 5, 7]]], np.float32)
    w = {"W1": None, "b1": None, "W2": np.array([[1, -1], [0, 0]], np.float32),
         "b2": np.array([ln3 + 2, 0], np.float32), "ws": np.array([0.5, -0.5, 4, 8], np.float32), "bs": ln3 - 4}
    d = _d(1, 2, 2, 1, 2, K=2, threshold=0.7)
    out = oracle.lookup(d, w, x)
    assert out["pooled"].tolist() == [[3.0, 5.0]]
    assert abs(out["logits"][0, 0] - out["logits"][0, 1] - ln3) < 1e-6
    assert abs(out["probs"][0, 0] - 0.75) < 1e-7 and out["pred_class"][0] == 0
    assert abs(out["score"][0] - ln3) < 1e-6 and abs(float(out["confidence"][0]) - 0.75) < 1e-6
    assert out["hit"][0] == 1


def test_pool_fc_lookup_against_library_ops(oracle):
    g = np.random.default_rng(5)
    n, C, ih, iw, oh, ow, K = 5, 6, 7, 7, 2, 2, 11
    F = C * oh * ow
    x = g.standard_normal((n, C, ih * iw)).astype(np.float32)
    w = {"W1": None, "b1": None, "W2": (g.standard_normal((K, F)) * 0.3).astype(np.float32),
         "b2": (g.standard_normal(K) * 0.1).astype(np.float32),
         "ws": (g.standard_normal(F + K) * 0.5).astype(np.float32), "bs": -0.2}
    d = _d(C, ih, iw, oh, ow, K=K, threshold=0.5)
    out = oracle.lookup(d, w, x)
    f = torch.relu(torch.nn.functional.adaptive_avg_pool2d(torch.from_numpy(x).double().reshape(n, C, ih, iw), (oh, ow)))
    f = f.reshape(n, F).float().double()
    z = f @ torch.from_numpy(w["W2"]).double().T + torch.from_numpy(w["b2"]).double()
    q = torch.softmax(z, dim=1)
    u = torch.cat([f, q], dim=1) @ torch.from_numpy(w["ws"]).double() + float(np.float32(-0.2))
    assert np.allclose(out["logits"], z.numpy(), atol=1e-5)
    assert np.allclose(out["score"], u.numpy(), atol=1e-5)
    assert np.array_equal(out["pred_class"], z.argmax(dim=1).numpy())
    # bf16 operand arithmetic: features and W2 rounded to bf16 before the products
    xb = torch.from_numpy(x).bfloat16()
    bits = xb.view(torch.int16).numpy().view(np.uint16)
    db = _d(C, ih, iw, oh, ow, K=K, dtype="bf16", threshold=0.5, round_operands=True)
    ob = oracle.lookup(db, w, bits)
    fb = torch.relu(torch.nn.functional.adaptive_avg_pool2d(xb.double().reshape(n, C, ih, iw), (oh, ow))).reshape(n, F).float()
    zb = fb.bfloat16().double() @ torch.from_numpy(w["W2"]).bfloat16().double().T + torch.from_numpy(w["b2"]).double()
    assert np.allclose(ob["logits"], zb.numpy(), atol=1e-5)


def test_adaptive_pool_channels_last(oracle):
    """The same map stored [position][channel]: identical features, bit for bit; a hand case in
    which a wrong stride would show; the library's channels-last pooling as a third opinion."""
    # 2 channels, 2x2 map -> 1x2.  channel-major rows: c0 = (1,2,3,4), c1 = (10,20,30,40);
    # channels-last the row reads (1,10, 2,20, 3,30, 4,40)
    x_ncs = np.array([[[1, 2, 3, 4], [10, 20, 30, 40]]], np.float32)
    x_nsc = np.array([[[1, 10], [2, 20], [3, 30], [4, 40]]], np.float32)
    want = [[2.0, 3.0, 20.0, 30.0]]                          # columns: (1+3)/2, (2+4)/2, (10+30)/2, (20+40)/2
    assert oracle.pool(_d(2, 2, 2, 1, 2), x_ncs).tolist() == want
    assert oracle.pool(_d(2, 2, 2, 1, 2, layout="nsc"), x_nsc).tolist() == want
    g = np.random.default_rng(5)
    for (C, ih, iw, oh, ow) in [(3, 7, 7, 2, 2), (4, 5, 9, 3, 2), (6, 14, 14, 4, 4)]:
        x = g.standard_normal((2, C, ih * iw)).astype(np.float32)
        xt = np.ascontiguousarray(x.transpose(0, 2, 1))
        a = oracle.pool(_d(C, ih, iw, oh, ow), x)
        b = oracle.pool(_d(C, ih, iw, oh, ow, layout="nsc"), xt)
        assert np.array_equal(a, b), (C, ih, iw)
        t = torch.from_numpy(x).double().reshape(2, C, ih, iw).contiguous(memory_format=torch.channels_last)
        ref = torch.relu(torch.nn.functional.adaptive_avg_pool2d(t, (oh, ow))).reshape(2, -1).numpy()
        assert np.allclose(b, ref, rtol=0, atol=1e-6)
