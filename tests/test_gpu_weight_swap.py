"""Retrained weights go from a trainer into a serving cache on the device (Section 5, retraining while
serving goes on): the cache must then answer exactly as one that received the same weights through
the host."""
import numpy as np
import pytest
import torch

import paper_2101_07344_amd as g

pytestmark = pytest.mark.gpu


def _f32(w):
    return {k: (np.asarray(v, np.float32) if k != "bs" else float(np.float32(v))) for k, v in w.items()}


def _weights(rng, predictor, selector, C, S, H, K, F, Hs, conv_k):
    w = {}
    if predictor == "gap_mlp":
        w["W1"], fin = rng.standard_normal((H, C)) * np.sqrt(2.0 / C), H
    elif predictor == "fc_mlp":
        w["W1"], fin = rng.standard_normal((H, C * S)) * np.sqrt(2.0 / (C * S)), H
    elif predictor == "conv_fc":
        w["W1"], fin = rng.standard_normal((H, C, conv_k, conv_k)) * np.sqrt(2.0 / (C * conv_k * conv_k)), F
    else:
        fin = F
    if predictor != "pool_fc":
        w["b1"] = rng.standard_normal(H) * 0.1
    w["W2"] = rng.standard_normal((K, fin)) * np.sqrt(2.0 / fin)
    w["b2"] = rng.standard_normal(K) * 0.1
    if selector == "linear":
        w["ws"], w["bs"] = rng.standard_normal(F + K) * 0.3, 0.1
    elif selector == "hidden":
        w["Ws"], w["cs"] = rng.standard_normal((Hs, F + K)) * 0.3, rng.standard_normal(Hs) * 0.1
        w["vs"], w["bs"] = rng.standard_normal(Hs) * 0.5, 0.1
    return _f32(w)


CASES = [
    # predictor, selector, dtype, layout, C, (ih, iw), H, K, n, extra
    ("gap_mlp", "linear", "bf16", "ncs", 72, (7, 7), 40, 10, 70, {}),
    ("gap_mlp", "linear", "f32", "nsc", 20, (5, 4), 33, 100, 50, {}),
    ("gap_mlp", "hidden", "bf16", "nsc", 64, (4, 4), 64, 37, 45, {}),
    ("gap_mlp", "softmax", "bf16", "ncs", 24, (6, 6), 16, 5, 33, {}),
    ("pool_fc", "linear", "bf16", "ncs", 16, (8, 8), 0, 10, 40, {"out_hw": (2, 2)}),
    ("pool_fc", "hidden", "f32", "ncs", 8, (6, 6), 0, 12, 40, {"out_hw": (3, 3)}),
    ("fc_mlp", "linear", "bf16", "ncs", 8, (4, 4), 48, 10, 60, {}),
    ("fc_mlp", "hidden", "f32", "ncs", 16, (2, 2), 40, 9, 33, {}),
    ("fc_mlp", "linear", "bf16", "ncs", 3, (5, 5), 20, 7, 25, {}),          # row length not a multiple of 64
    ("conv_fc", "linear", "bf16", "ncs", 8, (10, 10), 8, 12, 50, {"conv_ks": (3, 1)}),
    ("conv_fc", "hidden", "f32", "ncs", 4, (9, 8), 5, 6, 20, {"conv_ks": (3, 2)}),
    ("conv_fc", "softmax", "bf16", "nsc", 16, (6, 6), 4, 10, 30, {"conv_ks": (5, 1)}),
]


@pytest.mark.parametrize("predictor,selector,dtype,layout,C,hw,H,K,n,extra", CASES)
def test_device_side_swap_equals_the_host_path(predictor, selector, dtype, layout, C, hw, H, K, n, extra):
    rng = np.random.default_rng(1000 * C + 10 * K + len(predictor) + len(selector))
    ih, iw = hw
    S = ih * iw
    Hs = 12 if selector == "hidden" else 0
    conv_ks = extra.get("conv_ks", (0, 0))
    out_hw = extra.get("out_hw", (0, 0))
    if predictor == "pool_fc":
        F = C * out_hw[0] * out_hw[1]
    elif predictor == "conv_fc":
        F = H * ((ih - conv_ks[0]) // conv_ks[1] + 1) * ((iw - conv_ks[0]) // conv_ks[1] + 1)
    else:
        F = H if predictor == "fc_mlp" else C
    w_start = _weights(rng, predictor, selector, C, S, H, K, F, Hs, conv_ks[0])
    w_other = _weights(rng, predictor, selector, C, S, H, K, F, Hs, conv_ks[0])

    tr = g.Trainer(C, H, K, w_start, max_rows=n, sel_hidden=Hs, predictor=predictor, out_hw=out_hw, S=S, in_hw=hw,
                   conv_ks=conv_ks, selector=selector)
    # two steps so that the trainer holds weights nobody ever handed over through the host
    x = np.maximum(rng.standard_normal((n, tr.C)) + 0.2, 0).astype(np.float32)
    labels = torch.from_numpy(rng.integers(0, K, n).astype(np.int32)).cuda()
    Y = rng.random((n, K)).astype(np.float32) + 0.05
    Y = torch.from_numpy(Y / Y.sum(axis=1, keepdims=True)).cuda()
    xd = torch.from_numpy(x).cuda()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for _ in range(2):
            tr.step(xd, labels, Y, 0.05, 0.5, 2.0, stream=st)
    kw = dict(selector=selector, predictor=predictor, in_hw=hw, out_hw=out_hw, sel_hidden=Hs, conv_ks=conv_ks)
    swapped = g.Cache(C, S, H, K, dtype, layout, 0.5, n, w_other, **kw)
    # enqueued behind the steps on the same stream: the swap must see their result
    swapped.load_trainer(tr, stream=st)
    st.synchronize()
    trained = tr.get_weights()
    assert any(not np.array_equal(trained[k], w_start[k]) for k in ("W2", "b2"))
    through_host = g.Cache(C, S, H, K, dtype, layout, 0.5, n, trained, **kw)

    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    a = torch.from_numpy(np.maximum(rng.standard_normal((n, C, S)) + 0.3, 0).astype(np.float32)).cuda().to(tdt)
    act = a.permute(0, 2, 1).contiguous() if layout == "nsc" else a
    outs = []
    for cache in (swapped, through_host):
        pc = torch.full((n,), -7, dtype=torch.int32, device="cuda")
        conf = torch.full((n,), -7.0, device="cuda")
        hit = torch.full((n,), 9, dtype=torch.uint8, device="cuda")
        logits = torch.full((n, K), -7.0, device="cuda")
        cache.lookup(act, None, n, None, pc, conf, hit, logits)
        torch.cuda.synchronize()
        outs.append((pc.cpu().numpy(), conf.cpu().numpy(), hit.cpu().numpy(), logits.cpu().numpy()))
    for got, want, what in zip(outs[0], outs[1], ("pred_class", "confidence", "hit", "logits")):
        assert np.array_equal(got, want), what
    assert np.isfinite(outs[0][3]).all() and np.isfinite(outs[0][1]).all()
    tr.close(); swapped.close(); through_host.close()


def test_swap_refuses_a_trainer_of_another_shape():
    rng = np.random.default_rng(1)
    C, S, H, K, n = 16, 9, 24, 6, 8
    w = _weights(rng, "gap_mlp", "linear", C, S, H, K, C, 0, 0)
    cache = g.Cache(C, S, H, K, "bf16", "ncs", 0.5, n, w)
    for (C2, H2, K2, sel) in [(C, H + 8, K, "linear"), (C + 8, H, K, "linear"), (C, H, K + 1, "linear"), (C, H, K, "softmax")]:
        w2 = _weights(rng, "gap_mlp", sel, C2, S, H2, K2, C2, 0, 0)
        tr = g.Trainer(C2, H2, K2, w2, max_rows=n, selector=sel)
        with pytest.raises(g.GatiError):
            cache.load_trainer(tr)
        tr.close()
    wp = _weights(rng, "pool_fc", "linear", 4, S, 0, K, C, 0, 0)
    tr = g.Trainer(4, 0, K, wp, max_rows=n, predictor="pool_fc", out_hw=(2, 2))   # 16 features, but no hidden layer
    with pytest.raises(g.GatiError):
        cache.load_trainer(tr)
    tr.close(); cache.close()
