"""GPU parity of the paper's Conv(k,s) predictor: convolution -> ReLU -> FC."""
import numpy as np
import pytest
import torch

import oracle
import paper_2101_07344_amd as g
import workloads as W
from oracle import CacheDef, admit

from helpers import compare_lookup, ideal_def

pytestmark = pytest.mark.gpu

SHAPES = [
    # C, ih, iw, Co, k, s, K, n, dtype, variant
    (32, 14, 14, 8, 3, 1, 10, 40, "bf16", "conv_rows"),     # few filters: input-row formulation, 4-tap slots
    (16, 40, 40, 16, 3, 1, 7, 9, "bf16", "conv_mfma"),      # banded staging (S > 1024), ragged last band
    (16, 56, 56, 8, 5, 2, 12, 6, "bf16", "conv_rows"),      # Conv(5,2) on a ResNet stage-1 sized map: 14 tiles per wave
    (32, 9, 11, 40, 2, 1, 5, 21, "bf16", "conv_mfma"),      # 40 filters: two filter tiles, odd map
    (16, 12, 12, 5, 3, 2, 6, 33, "f32", "conv_mfma"),       # fp32 MFMA, 8-channel blocks
    (16, 6, 6, 4, 6, 1, 4, 17, "bf16", "conv_mfma"),        # filter as large as the map: one output pixel
    (64, 7, 7, 8, 1, 1, 9, 12, "bf16", "conv_rows"),        # 1x1 filter, odd plane size
    (12, 10, 10, 3, 3, 1, 4, 11, "bf16", "conv_generic"),   # channels not a whole block
    (5, 9, 7, 2, 4, 3, 3, 8, "f32", "conv_generic"),
    (32, 32, 40, 4, 3, 1, 6, 5, "bf16", "conv_mfma"),       # wide rows: 38 output columns, several bands
    (32, 28, 28, 8, 5, 2, 10, 7, "bf16", "conv_rows"),      # two input rows per tile
    (32, 28, 28, 16, 5, 2, 10, 7, "bf16", "conv_mfma"),     # 16 filters: whole-plane staging with the transposing store
    (16, 16, 16, 40, 3, 1, 6, 9, "bf16", "conv_mfma"),      # the same with two filter tiles
    (16, 24, 24, 8, 3, 1, 5, 6, "f32", "conv_mfma"),        # fp32, several tiles per wave
    # the input-row kernel: every slot width, parity, wave split and fill shape
    (2048, 7, 7, 8, 3, 1, 10, 30, "bf16", "conv_rows"),     # 7x7 planes of 98 bytes: odd fragment starts, channel parts, 16 fills
    (1024, 14, 14, 8, 3, 1, 10, 9, "bf16", "conv_rows"),    # few rows: the channels of a request shared among workgroups
    (64, 30, 30, 7, 7, 2, 6, 5, "bf16", "conv_rows"),       # Conv(7,2): four tap rows per parity, 7 filters
    (32, 18, 16, 8, 4, 2, 6, 5, "bf16", "conv_rows"),       # even filter, non-square map
    (16, 13, 11, 5, 3, 2, 6, 12, "bf16", "conv_rows"),      # odd row length with stride 2: 4-tap slots, odd starts
    (24, 9, 33, 2, 2, 1, 4, 7, "bf16", "conv_rows"),        # 32 output columns: every pixel lane of a tile in use
    (8, 20, 21, 1, 3, 1, 3, 6, "bf16", "conv_rows"),        # one filter, 19 columns in 32 lanes
    (16, 12, 10, 6, 3, 2, 5, 14, "bf16", "conv_generic:nsc"),   # channels-last map
    (7, 9, 9, 3, 2, 1, 4, 10, "f32", "conv_generic:nsc"),
]


def _weights(C, Co, k, K, F, rng):
    return {"W1": (rng.standard_normal((Co, C, k, k)) * np.sqrt(2 / (C * k * k))).astype(np.float32),
            "b1": (rng.standard_normal(Co) * 0.1).astype(np.float32),
            "W2": (rng.standard_normal((K, F)) * np.sqrt(2 / F)).astype(np.float32),
            "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
            "ws": (rng.standard_normal(F + K) * np.sqrt(2 / (F + K))).astype(np.float32), "bs": 0.0}


@pytest.mark.parametrize("C,ih,iw,Co,k,s,K,n,dtype,variant", SHAPES)
def test_conv_predictor_matches_oracle(C, ih, iw, Co, k, s, K, n, dtype, variant):
    rng = np.random.default_rng(C * ih + Co * k + s)
    S = ih * iw
    variant, _, layout = variant.partition(":")
    layout = layout or "ncs"
    x = torch.from_numpy((rng.standard_normal((n, C, S) if layout == "ncs" else (n, S, C)) + 0.2).astype(np.float32))
    x = x.bfloat16() if dtype == "bf16" else x
    d = CacheDef(C=C, S=S, H=Co, K=K, dtype=dtype, threshold=0.5, round_operands=(dtype == "bf16"),
                 predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s), layout=layout)
    F = d.F
    w = _weights(C, Co, k, K, F, rng)
    host = W.to_host_array(x)
    s0 = oracle.lookup(d, w, host)["score"]
    w["bs"] = float(np.float32(-np.median(s0)))
    ok = np.setdiff1d(np.arange(n), admit.inadmissible_rows(d, w, host)).astype(np.int32)
    assert len(ok) > n // 2
    want = oracle.lookup(d, w, host, row_index=ok)
    cache = g.Cache(C, S, Co, K, dtype, layout, 0.5, n, w, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
    assert cache.pool_variant == variant and cache.F == F
    m = len(ok)
    okd = torch.from_numpy(ok).cuda()
    xd = x.cuda()
    # the hidden layer alone
    feat = torch.full((m, F), -1.0, device="cuda")
    cache.pool(xd, okd, m, None, feat)
    torch.cuda.synchronize()
    err = np.max(np.abs(feat.cpu().numpy() - want["pooled"]))
    assert err <= (2e-3 if dtype == "bf16" else 1e-4), err
    out = {"pred_class": torch.zeros(m, dtype=torch.int32, device="cuda"), "confidence": torch.zeros(m, device="cuda"),
           "hit": torch.zeros(m, dtype=torch.uint8, device="cuda"), "logits": torch.zeros(m, K, device="cuda")}
    ids_out = torch.zeros(m, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    cache.lookup_compact(xd, okd, m, None, out["pred_class"], out["confidence"], out["hit"], out["logits"],
                         okd, ids_out, cnt)
    torch.cuda.synchronize()
    got = {key: v.cpu().numpy() for key, v in out.items()}
    want_ideal = oracle.lookup(ideal_def(d), w, host, row_index=ok) if dtype == "bf16" else None
    compare_lookup(got, want, want_ideal, dtype, f"conv {C}x{ih}x{iw} k{k}s{s} -> {Co}")
    want_ids = oracle.compact_misses(want["hit"], ok)
    assert int(cnt.item()) == len(want_ids)
    assert np.array_equal(ids_out.cpu().numpy()[:len(want_ids)], want_ids)
    # device-side count below n_max: rows past it stay untouched; same bits for the rest
    n_dev = torch.tensor([m // 2], dtype=torch.int32, device="cuda")
    feat2 = torch.full((m, F), -7.0, device="cuda")
    cache.pool(xd, okd, m, n_dev, feat2)
    torch.cuda.synchronize()
    f2 = feat2.cpu().numpy()
    assert np.array_equal(f2[:m // 2], feat.cpu().numpy()[:m // 2]) and np.all(f2[m // 2:] == -7.0)
    cache.close()


@pytest.mark.parametrize("C,ih,iw,k,s", [(64, 56, 56, 5, 2), (128, 28, 28, 5, 2), (256, 14, 14, 3, 1), (512, 7, 7, 3, 1)])
def test_conv_rows_many_fills_per_workgroup(C, ih, iw, k, s):
    """A cache sized for a large batch keeps all channels of a request in one workgroup: 16 and more
    fills run through every slot of the LDS ring, as in the full-size stacks, here against the oracle
    on every hidden value."""
    rng = np.random.default_rng(C + ih)
    n, Co, K, S = 6, 8, 5, ih * iw
    x = torch.from_numpy((rng.standard_normal((n, C, S)) + 0.2).astype(np.float32)).bfloat16()
    d = CacheDef(C=C, S=S, H=Co, K=K, dtype="bf16", threshold=0.5, round_operands=True,
                 predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
    w = _weights(C, Co, k, K, d.F, rng)
    want = oracle.lookup(d, w, W.to_host_array(x))["pooled"]
    cache = g.Cache(C, S, Co, K, "bf16", "ncs", 0.5, 512, w, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
    assert cache.pool_variant == "conv_rows"
    feat = torch.full((n, d.F), -1.0, device="cuda")
    cache.pool(x.cuda(), None, n, None, feat)
    torch.cuda.synchronize()
    err = np.max(np.abs(feat.cpu().numpy() - want))
    assert err <= 2e-3, err
    cache.close()


def test_conv_rejects_bad_shapes():
    def make(C, ih, iw, Co, k, s, layout="ncs", S=None):
        oh, ow = max(0, (ih - k) // s + 1), max(0, (iw - k) // s + 1)
        F = Co * oh * ow
        w = {"W1": np.zeros((Co, C, k, k), np.float32), "b1": np.zeros(Co, np.float32),
             "W2": np.zeros((3, F), np.float32), "b2": np.zeros(3, np.float32), "ws": np.zeros(F + 3, np.float32), "bs": 0.0}
        return g.Cache(C, S or ih * iw, Co, 3, "f32", layout, 0.5, 4, w, predictor="conv_fc", in_hw=(ih, iw), conv_ks=(k, s))
    with pytest.raises(g.GatiError):       # filter larger than the map
        make(8, 3, 3, 4, 4, 1)
    with pytest.raises(g.GatiError):       # more filters than the kernels hold
        make(8, 4, 4, 65, 3, 1)
    make(8, 4, 4, 64, 3, 1).close()
