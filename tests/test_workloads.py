"""The seeded input generators: shapes, distributions, reproducibility."""
import numpy as np
import torch

import workloads as W


def test_zipf_labels_follow_the_power_law():
    lab = W.zipf_labels(200000, 10, 1.1, seed=0)
    assert lab.dtype == np.int32 and lab.min() == 0 and lab.max() == 9
    freq = np.bincount(lab, minlength=10) / len(lab)
    pmf = np.arange(1, 11, dtype=np.float64) ** -1.1
    pmf /= pmf.sum()
    assert np.max(np.abs(freq - pmf)) < 5e-3
    assert np.array_equal(lab, W.zipf_labels(200000, 10, 1.1, seed=0))
    assert not np.array_equal(lab, W.zipf_labels(200000, 10, 1.1, seed=1))


def test_directions_and_weights():
    spec = W.get_workload("tiny")
    d = W.class_directions(spec, 0)
    assert d.shape == (10, 64) and np.allclose(np.linalg.norm(d, axis=1), 1.0, atol=1e-6)
    w = W.cache_weights(spec, 0)
    assert w["W1"].shape == (128, 64) and w["W2"].shape == (10, 128) and w["ws"].shape == (74,)
    assert abs(w["W1"].std() - np.sqrt(2 / 64)) < 0.01
    assert abs(w["W2"].std() - np.sqrt(2 / 128)) < 0.02
    assert not w["b1"].any() and not w["b2"].any()
    assert np.array_equal(w["W1"], W.cache_weights(spec, 0)["W1"])


def test_workload_shapes_match_the_configs():
    r18, r50, bert, r152 = (W.get_workload(n) for n in ("resnet18", "resnet50", "bert_base", "resnet152"))
    assert [(l.C, l.S) for l in r18.layers] == [(64, 3136)] * 2 + [(128, 784)] * 2 + [(256, 196)] * 2 + [(512, 49)] * 2
    assert r18.batch == 256 and all(l.dtype == "f32" and l.H == 256 and l.K == 1000 for l in r18.layers)
    assert len(r50.layers) == 16 and [l.C for l in r50.layers] == [256] * 3 + [512] * 4 + [1024] * 6 + [2048] * 3
    assert r50.batch == 512 and all(l.dtype == "bf16" and l.H == 512 for l in r50.layers)
    assert sum(l.row_bytes for l in r50.layers) * r50.batch == 5_651_824_640     # ~5.65 GB per stack
    assert len(bert.layers) == 12 and all((l.C, l.S, l.H, l.K, l.layout) == (768, 128, 256, 20, "nsc") for l in bert.layers)
    assert bert.batch == 1024 and bert.layers[0].row_bytes == 196608
    assert len(r152.layers) == 50 and r152.batch == 4096 and r152.storage == "dense"


def test_activation_rows_are_reproducible_per_row():
    spec = W.get_workload("tiny")
    lab = W.zipf_labels(spec.batch, 10, spec.zipf_s, spec.seed)
    a = W.activation_rows(spec, 0, lab, [0, 1, 2, 3])
    b = W.activation_rows(spec, 0, lab, [3, 1])
    assert a.shape == (4, 64, 64) and a.dtype == torch.float32 and a.min() >= 0
    assert torch.equal(a[3], b[0]) and torch.equal(a[1], b[1])
    c = W.activation_rows(spec, 0, lab, [3], attempts=[1])
    assert not torch.equal(c[0], a[3])
    # class means: the channel means follow gamma * d[label]
    L = spec.layers[0]
    big = W.activation_rows(spec, 0, lab, list(range(64)))
    assert abs(float(big.mean()) - 0.4) < 0.2             # E relu(N(mu,1)) ~ 0.40 + mu/2 for small mu


def test_bert_rows_are_token_major_bf16():
    spec = W.get_workload("bert_base").scaled(4)
    lab = W.zipf_labels(4, 20, spec.zipf_s, spec.seed)
    a = W.activation_rows(spec, 0, lab, [0, 1])
    assert a.shape == (2, 128, 768) and a.dtype == torch.bfloat16
    assert a.min() < 0                                     # no ReLU on token states
    h = W.to_host_array(a)
    assert h.dtype == np.uint16 and h.shape == (2, 128, 768)
    bulk = W.activation_bulk(spec, 0, lab, [0, 1, 2, 3], device="cpu")
    assert bulk.shape == (4, 128, 768)
    assert torch.equal(bulk, W.activation_bulk(spec, 0, lab, [0, 1, 2, 3], device="cpu"))


def test_variant_workloads_have_their_feature_counts_and_fitted_biases():
    want_F = {"resnet50_pool": [4096] * 3 + [8192] * 4 + [4096] * 6 + [8192] * 3,
              "resnet50_conv": [5408] * 3 + [1152] * 4 + [1152] * 6 + [200] * 3,
              "resnet50_fc": [1024] * 6, "resnet50_hsel": [256] * 3 + [512] * 4 + [1024] * 6 + [2048] * 3}
    for name, fs in want_F.items():
        spec = W.get_workload(name)
        assert [l.F for l in spec.layers] == fs, name
        assert all(l.target_hit is not None for l in spec.layers), name       # the stored calibration was applied
        assert len({round(l.bs, 6) for l in spec.layers}) > 1, name
        w = W.cache_weights(spec, len(spec.layers) - 1)
        L = spec.layers[-1]
        assert w["W2"].shape == (L.K, L.F if L.predictor in ("pool_fc", "conv_fc") else L.H)
        if L.selector == "hidden":
            assert w["Ws"].shape == (L.sel_hidden, L.F + L.K) and w["vs"].shape == (L.sel_hidden,)
            base = W.cache_weights(W.get_workload("resnet50"), len(spec.layers) - 1)
            assert np.array_equal(w["W1"], base["W1"])                          # same predictor as the linear stack
        if L.predictor == "conv_fc":
            assert w["W1"].shape == (L.H, L.C, L.conv_ks[0], L.conv_ks[0])
