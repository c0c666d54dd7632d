"""Pins for the convolution predictor (Section 3, table of predictor architectures:
Input -Conv-> Hidden Layer -FC-> Output, Conv(k,s) = kernel size and stride, ReLU)."""
import numpy as np
import torch

from oracle import CacheDef


def _w(C, Co, k, K, F, **kw):
    w = {"W1": np.zeros((Co, C, k, k), np.float32), "b1": np.zeros(Co, np.float32),
         "W2": np.zeros((K, F), np.float32), "b2": np.zeros(K, np.float32),
         "ws": np.zeros(F + K, np.float32), "bs": 0.0}
    for key, v in kw.items():
        w[key] = v if key == "bs" else np.asarray(v, np.float32)
    return w


def _features(oracle, d, w, x):
    return oracle.lookup(d, w, x)["pooled"]


def test_hand_case_2x2_filter_on_3x3_map(oracle):
    d = CacheDef(C=1, S=9, H=1, K=1, predictor="conv_fc", in_hw=(3, 3), conv_ks=(2, 1))
    assert d.F == 4
    x = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 9)          # rows (1,2,3), (4,5,6), (7,8,9)
    # 1*1+2*2+3*4+4*5 = 37;  1*2+2*3+3*5+4*6 = 47;  1*4+2*5+3*7+4*8 = 67;  1*5+2*6+3*8+4*9 = 77
    f = _features(oracle, d, _w(1, 1, 2, 1, 4, W1=[[[[1, 2], [3, 4]]]]), x)
    assert f.tolist() == [[37, 47, 67, 77]]
    # x[y,x] - x[y+1,x+1] = -4 everywhere: ReLU clamps it; a bias of 5 lifts it to 1
    f = _features(oracle, d, _w(1, 1, 2, 1, 4, W1=[[[[1, 0], [0, -1]]]]), x)
    assert f.tolist() == [[0, 0, 0, 0]]
    f = _features(oracle, d, _w(1, 1, 2, 1, 4, W1=[[[[1, 0], [0, -1]]]], b1=[5]), x)
    assert f.tolist() == [[1, 1, 1, 1]]


def test_index_order_and_stride_probe(oracle):
    """x[c,y,x] = 100c + 10y + x; a one-hot filter tap (o,c,dy,dx) must pick x[c, oy*s+dy, ox*s+dx],
    and filter o must land in feature block o (features are [o][oy][ox])."""
    C, ih, iw, Co = 3, 7, 8, 2
    x = np.array([[[100 * c + 10 * y + xx for y in range(ih) for xx in range(iw)] for c in range(C)]], np.float32)
    for k, s in ((3, 1), (3, 2), (5, 2), (2, 3)):
        oh, ow = (ih - k) // s + 1, (iw - k) // s + 1
        d = CacheDef(C=C, S=ih * iw, H=Co, K=1, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
        assert d.F == Co * oh * ow
        for (o, c, dy, dx) in ((0, 0, 0, 0), (1, 2, k - 1, 0), (0, 1, 1, k - 1), (1, 1, k - 1, k - 1)):
            W1 = np.zeros((Co, C, k, k), np.float32)
            W1[o, c, dy, dx] = 1.0
            f = _features(oracle, d, _w(C, Co, k, 1, d.F, W1=W1), x).reshape(Co, oh, ow)
            want = np.array([[100 * c + 10 * (oy * s + dy) + ox * s + dx for ox in range(ow)] for oy in range(oh)])
            assert np.array_equal(f[o], want), (k, s, o, c, dy, dx)
            assert not f[1 - o].any()


def test_against_library_convolution(oracle):
    rng = np.random.default_rng(11)
    for (C, ih, iw, Co, k, s) in ((4, 9, 7, 3, 3, 1), (5, 11, 11, 2, 5, 2), (2, 6, 10, 4, 2, 2), (3, 5, 5, 2, 1, 1)):
        d = CacheDef(C=C, S=ih * iw, H=Co, K=1, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
        x = rng.standard_normal((2, C, ih * iw)).astype(np.float32)
        W1 = rng.standard_normal((Co, C, k, k)).astype(np.float32)
        b1 = rng.standard_normal(Co).astype(np.float32)
        f = _features(oracle, d, _w(C, Co, k, 1, d.F, W1=W1, b1=b1), x)
        ref = torch.nn.functional.conv2d(torch.from_numpy(x.reshape(2, C, ih, iw)).double(),
                                         torch.from_numpy(W1).double(), torch.from_numpy(b1).double(), stride=s)
        ref = torch.relu(ref).reshape(2, -1).numpy()
        assert f.shape == ref.shape
        assert np.max(np.abs(f - ref)) < 1e-5 and np.array_equal(f, ref.astype(np.float32))


def test_full_size_filter_is_the_fully_connected_predictor(oracle):
    """k = in_h = in_w: one output position per filter, i.e. FC over the flattened row."""
    rng = np.random.default_rng(3)
    C, hw, Co, K = 3, 4, 5, 6
    x = rng.standard_normal((4, C, hw * hw)).astype(np.float32)
    W1 = rng.standard_normal((Co, C, hw, hw)).astype(np.float32)
    b1 = rng.standard_normal(Co).astype(np.float32)
    W2 = rng.standard_normal((K, Co)).astype(np.float32)
    ws = rng.standard_normal(Co + K).astype(np.float32)
    dc = CacheDef(C=C, S=hw * hw, H=Co, K=K, predictor="conv_fc", in_hw=(hw, hw), conv_ks=(hw, 1))
    df = CacheDef(C=C, S=hw * hw, H=Co, K=K, predictor="fc_mlp")
    a = oracle.lookup(dc, _w(C, Co, hw, K, Co, W1=W1, b1=b1, W2=W2, ws=ws, bs=0.1), x)
    b = oracle.lookup(df, {"W1": W1.reshape(Co, -1), "b1": b1, "W2": W2, "b2": np.zeros(K, np.float32), "ws": ws, "bs": 0.1}, x)
    for key in ("pooled", "logits", "confidence", "pred_class", "hit"):
        assert np.array_equal(a[key], b[key]), key


def test_lookup_feeds_the_conv_features_to_the_output_layer(oracle):
    rng = np.random.default_rng(8)
    C, ih, iw, Co, k, s, K = 3, 6, 6, 2, 3, 1, 4
    d = CacheDef(C=C, S=ih * iw, H=Co, K=K, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s), threshold=0.5)
    F = d.F
    x = rng.standard_normal((3, C, ih * iw)).astype(np.float32)
    w = _w(C, Co, k, K, F, W1=rng.standard_normal((Co, C, k, k)), b1=rng.standard_normal(Co),
           W2=rng.standard_normal((K, F)) * 0.2, b2=rng.standard_normal(K), ws=rng.standard_normal(F + K) * 0.1, bs=0.2)
    out = oracle.lookup(d, w, x)
    f = out["pooled"].astype(np.float64)
    z = f @ w["W2"].astype(np.float64).T + w["b2"]
    assert np.max(np.abs(out["logits"] - z)) < 1e-5
    q = np.exp(z - z.max(1, keepdims=True))
    q /= q.sum(1, keepdims=True)
    u = float(np.float32(0.2)) + f @ w["ws"][:F].astype(np.float64) + q @ w["ws"][F:].astype(np.float64)
    assert np.max(np.abs(out["score"] - u)) < 1e-9
    assert np.array_equal(out["pred_class"], z.argmax(1))


def test_bf16_arithmetic_rounds_the_filter(oracle):
    e = 2.0 ** -8          # 1 + 2^-8 is a tie between bf16 neighbours and rounds to 1
    d = CacheDef(C=1, S=4, H=1, K=1, predictor="conv_fc", in_hw=(2, 2), conv_ks=(2, 1), dtype="bf16", round_operands=True)
    x = np.array([[[0x4040, 0, 0, 0]]], np.uint16)            # 3.0 at (0,0)
    f = _features(oracle, d, _w(1, 1, 2, 1, 1, W1=[[[[1 + e, 0], [0, 0]]]]), x)
    assert f.tolist() == [[3.0]]
    d0 = CacheDef(C=1, S=4, H=1, K=1, predictor="conv_fc", in_hw=(2, 2), conv_ks=(2, 1), dtype="bf16")
    f0 = _features(oracle, d0, _w(1, 1, 2, 1, 1, W1=[[[[1 + e, 0], [0, 0]]]]), x)
    assert f0.tolist() == [[np.float32(3 * (1 + e))]]


def test_channels_last_map_gives_the_same_features(oracle):
    """The map stored [position][channel]: the index probe again (a wrong stride would pick another
    element), and equality with the channel-major result on random data."""
    C, ih, iw, Co, k, s = 3, 5, 6, 2, 3, 2
    oh, ow = (ih - k) // s + 1, (iw - k) // s + 1
    x = np.array([[[100 * c + 10 * y + xx for y in range(ih) for xx in range(iw)] for c in range(C)]], np.float32)
    xt = np.ascontiguousarray(x.transpose(0, 2, 1))
    d_ncs = CacheDef(C=C, S=ih * iw, H=Co, K=1, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
    d_nsc = CacheDef(C=C, S=ih * iw, H=Co, K=1, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s), layout="nsc")
    for (o, c, dy, dx) in ((0, 0, 0, 0), (1, 2, k - 1, 1), (0, 1, 1, k - 1)):
        W1 = np.zeros((Co, C, k, k), np.float32)
        W1[o, c, dy, dx] = 1.0
        f = _features(oracle, d_nsc, _w(C, Co, k, 1, d_nsc.F, W1=W1), xt).reshape(Co, oh, ow)
        want = np.array([[100 * c + 10 * (oy * s + dy) + ox * s + dx for ox in range(ow)] for oy in range(oh)])
        assert np.array_equal(f[o], want) and not f[1 - o].any()
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, C, ih * iw)).astype(np.float32)
    w = _w(C, Co, k, 1, d_ncs.F, W1=rng.standard_normal((Co, C, k, k)), b1=rng.standard_normal(Co))
    assert np.array_equal(_features(oracle, d_ncs, w, x), _features(oracle, d_nsc, w, np.ascontiguousarray(x.transpose(0, 2, 1))))
