"""Seeded sweep of valid shapes through every feature-stage kernel family: whatever variant the
library plans for a shape, the features must match the oracle's (sizes stay small enough for the
oracle to finish in seconds)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2101_07344_amd as g
import workloads as W
from oracle import CacheDef

pytestmark = pytest.mark.gpu


def _features_match(d, w, x, cache, n, tol):
    host = W.to_host_array(x)
    want = oracle.lookup(d, w, host)["pooled"]
    got = torch.full((n, d.F), -5.0, device="cuda")
    cache.pool(x.cuda(), None, n, None, got)
    torch.cuda.synchronize()
    err = float(np.max(np.abs(got.cpu().numpy() - want))) if want.size else 0.0
    assert err <= tol, (cache.pool_variant, err)


def _zero_head(F, K, H=None, W1=None):
    return {"W1": W1, "b1": None if W1 is None else np.zeros(W1.shape[0], np.float32),
            "W2": np.zeros((K, F if H is None else H), np.float32), "b2": np.zeros(K, np.float32),
            "ws": np.zeros(F + K, np.float32), "bs": 0.0}


def test_global_pool_random_shapes():
    rng = np.random.default_rng(2024)
    seen = set()
    for _ in range(40):
        layout = "ncs" if rng.random() < 0.6 else "nsc"
        dtype = "bf16" if rng.random() < 0.6 else "f32"
        C = int(rng.choice([1, 3, 8, 24, 40, 64, 96, 130, 256, 520]))
        S = int(rng.choice([1, 2, 7, 16, 33, 49, 64, 100, 196, 257, 784]))
        n = int(rng.integers(1, 12))
        x = torch.from_numpy(rng.standard_normal((n, C, S) if layout == "ncs" else (n, S, C)).astype(np.float32))
        x = x.bfloat16() if dtype == "bf16" else x
        d = CacheDef(C=C, S=S, H=4, K=3, dtype=dtype, layout=layout)
        w = _zero_head(C, 3, H=4, W1=np.zeros((4, C), np.float32))
        cache = g.Cache(C, S, 4, 3, dtype, layout, 0.5, n, w)
        seen.add(cache.pool_variant)
        _features_match(d, w, x, cache, n, 2e-6 * max(1.0, float(x.float().abs().max())))
        cache.close()
    assert {"ncs_wave", "ncs_segw", "generic"} <= seen and ({"nsc_unit", "nsc_vec"} & seen)


def test_adaptive_pool_random_shapes():
    rng = np.random.default_rng(7)
    seen = set()
    for _ in range(30):
        dtype = "bf16" if rng.random() < 0.6 else "f32"
        C = int(rng.choice([4, 8, 16, 40, 64, 128]))
        ih, iw = int(rng.integers(1, 30)), int(rng.integers(1, 30))
        oh, ow = int(rng.integers(1, ih + 1)), int(rng.integers(1, iw + 1))
        if C * oh * ow > 4096:
            oh, ow = max(1, oh // 4), max(1, ow // 4)
        n = int(rng.integers(1, 7))
        x = torch.from_numpy(rng.standard_normal((n, C, ih * iw)).astype(np.float32))
        x = x.bfloat16() if dtype == "bf16" else x
        F = C * oh * ow
        d = CacheDef(C=C, S=ih * iw, H=0, K=3, dtype=dtype, predictor="pool_fc", in_hw=(ih, iw), out_hw=(oh, ow))
        w = _zero_head(F, 3)
        cache = g.Cache(C, ih * iw, 0, 3, dtype, "ncs", 0.5, n, w, predictor="pool_fc", in_hw=(ih, iw), out_hw=(oh, ow))
        seen.add(cache.pool_variant)
        _features_match(d, w, x, cache, n, 2e-6 * max(1.0, float(x.float().abs().max())))
        cache.close()
    assert seen == {"ncs_adaptive", "adaptive_generic"}


def test_conv_random_shapes():
    rng = np.random.default_rng(99)
    seen = set()
    for _ in range(40):
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        C = int(rng.choice([8, 16, 32, 48, 12]))
        ih, iw = int(rng.integers(3, 41)), int(rng.integers(3, 41))
        if rng.random() < 0.5:
            iw = int(rng.choice([8, 16, 24, 40]))         # widths the banded / transposing paths accept
        k = int(rng.integers(1, min(ih, iw, 6) + 1))
        s = int(rng.integers(1, 4))
        Co = int(rng.choice([1, 4, 8, 33]))
        n = int(rng.integers(1, 5))
        S = ih * iw
        x = torch.from_numpy((rng.standard_normal((n, C, S)) + 0.1).astype(np.float32))
        x = x.bfloat16() if dtype == "bf16" else x
        d = CacheDef(C=C, S=S, H=Co, K=3, dtype=dtype, round_operands=(dtype == "bf16"), predictor="conv_fc",
                     in_hw=(ih, iw), conv_ks=(k, s))
        W1 = (rng.standard_normal((Co, C, k, k)) * np.sqrt(2 / (C * k * k))).astype(np.float32)
        w = _zero_head(d.F, 3, W1=W1)
        w["W2"] = np.zeros((3, d.F), np.float32)
        w["b1"] = (rng.standard_normal(Co) * 0.1).astype(np.float32)
        cache = g.Cache(C, S, Co, 3, dtype, "ncs", 0.5, n, w, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
        seen.add(cache.pool_variant)
        _features_match(d, w, x, cache, n, 4e-3 if dtype == "bf16" else 2e-4)
        cache.close()
    assert seen == {"conv_mfma", "conv_generic", "conv_rows"}


def test_lookup_random_head_shapes():
    """Random widths through the FC / softmax / selector / finish kernels (tile-ragged H, K, n)."""
    from oracle import admit
    from helpers import compare_lookup, ideal_def
    rng = np.random.default_rng(31)
    for trial in range(16):
        dtype = "bf16" if trial % 2 else "f32"
        selector = ("linear", "softmax", "hidden")[trial % 3]
        C = int(rng.choice([5, 32, 70, 128, 300]))
        S = int(rng.choice([4, 9, 16]))
        H = int(rng.integers(1, 200))
        K = int(rng.integers(2, 260))
        Hs = int(rng.integers(1, 70))
        n = int(rng.integers(1, 100))
        x = torch.from_numpy(np.maximum(rng.standard_normal((n, C, S)) + 0.3, 0).astype(np.float32))
        x = x.bfloat16() if dtype == "bf16" else x
        w = {"W1": (rng.standard_normal((H, C)) * np.sqrt(2 / C)).astype(np.float32),
             "b1": (rng.standard_normal(H) * 0.1).astype(np.float32),
             "W2": (rng.standard_normal((K, H)) * np.sqrt(2 / H)).astype(np.float32),
             "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
             "ws": (rng.standard_normal(C + K) * 2 * np.sqrt(2 / (C + K))).astype(np.float32), "bs": 0.0,
             "Ws": (rng.standard_normal((Hs, C + K)) * 4 * np.sqrt(2 / (C + K))).astype(np.float32),
             "cs": (rng.standard_normal(Hs) * 0.1).astype(np.float32),
             "vs": (rng.standard_normal(Hs) * np.sqrt(2 / Hs)).astype(np.float32)}
        host = W.to_host_array(x)
        d = CacheDef(C=C, S=S, H=H, K=K, dtype=dtype, threshold=0.5, round_operands=(dtype == "bf16"),
                     selector=selector, sel_hidden=Hs if selector == "hidden" else 0)
        if selector == "softmax":
            d.threshold = float(np.float32(np.median(oracle.lookup(d, w, host)["confidence"])))
        else:
            w["bs"] = float(np.float32(-np.median(oracle.lookup(d, w, host)["score"])))
        ok = np.setdiff1d(np.arange(n), admit.inadmissible_rows(d, w, host)).astype(np.int32)
        if len(ok) == 0:
            continue
        want = oracle.lookup(d, w, host, row_index=ok)
        cache = g.Cache(C, S, H, K, dtype, "ncs", d.threshold, n, w, selector=selector, sel_hidden=d.sel_hidden)
        m = len(ok)
        out = {"pred_class": torch.zeros(m, dtype=torch.int32, device="cuda"), "confidence": torch.zeros(m, device="cuda"),
               "hit": torch.zeros(m, dtype=torch.uint8, device="cuda"), "logits": torch.zeros(m, K, device="cuda")}
        ids_out = torch.zeros(m, dtype=torch.int32, device="cuda")
        cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        okd = torch.from_numpy(ok).cuda()
        cache.lookup_compact(x.cuda(), okd, m, None, out["pred_class"], out["confidence"], out["hit"], out["logits"],
                             okd, ids_out, cnt)
        torch.cuda.synchronize()
        got = {key: v.cpu().numpy() for key, v in out.items()}
        want_ideal = oracle.lookup(ideal_def(d), w, host, row_index=ok) if dtype == "bf16" else None
        # against unrounded arithmetic the bf16 gap scales with the logits (2^-9 relative per operand):
        # the 2e-2 bound is stated for logits of a few units, as in the workloads
        scale = max(1.0, float(np.max(np.abs(want["logits"]))) / 4.0)
        compare_lookup(got, want, want_ideal, dtype, f"trial {trial}: {C}x{S}->{H}->{K} {selector} {dtype} n={n}",
                       tol_ideal=2e-2 * scale)
        want_ids = oracle.compact_misses(want["hit"], ok)
        assert int(cnt.item()) == len(want_ids) and np.array_equal(ids_out.cpu().numpy()[:len(want_ids)], want_ids)
        cache.close()
