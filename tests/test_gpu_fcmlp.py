"""GPU parity of the paper's FC(h) predictor: flattened activation -> FC -> ReLU -> FC."""
import numpy as np
import pytest
import torch

import oracle
import paper_2101_07344_amd as g
import workloads as W
from oracle import CacheDef, admit

from helpers import compare_lookup, ideal_def

pytestmark = pytest.mark.gpu


def _weights(D, H, K, rng):
    return {"W1": (rng.standard_normal((H, D)) * np.sqrt(2 / D)).astype(np.float32),
            "b1": (rng.standard_normal(H) * 0.05).astype(np.float32),
            "W2": (rng.standard_normal((K, H)) * np.sqrt(2 / H)).astype(np.float32),
            "b2": (rng.standard_normal(K) * 0.1).astype(np.float32),
            "ws": (rng.standard_normal(H + K) * np.sqrt(2 / (H + K))).astype(np.float32), "bs": 0.0}


@pytest.mark.parametrize("C,S,H,K,n,dtype,layout", [
    (8, 16, 40, 7, 45, "bf16", "ncs"),        # 1x1 wave tiles, one split
    (64, 64, 128, 33, 150, "f32", "ncs"),     # 2x2 wave tiles, fp32 MFMA
    (32, 196, 256, 100, 300, "bf16", "ncs"),  # 4x4 wave tiles, several splits, ragged rows
    (48, 64, 256, 20, 260, "bf16", "nsc"),    # token-major storage: flattened as stored
    (48, 50, 256, 20, 260, "bf16", "nsc"),    # D = 2400, not a multiple of 64: the plain kernel
    (5, 7, 8, 3, 40, "f32", "ncs"),           # D = 35, H a multiple of nothing useful
    (33, 49, 70, 11, 90, "bf16", "ncs"),      # odd everything, bf16
    (16, 72, 256, 12, 270, "f32", "ncs"),     # 4x4 wave tiles through LDS, fp32 MFMA, odd stage count
])
def test_fc_mlp_lookup_matches_oracle(C, S, H, K, n, dtype, layout):
    rng = np.random.default_rng(C * S + H)
    D = C * S
    shape = (n, C, S) if layout == "ncs" else (n, S, C)
    x = torch.from_numpy(np.maximum(rng.standard_normal(shape) + 0.3, 0).astype(np.float32))
    x = x.bfloat16() if dtype == "bf16" else x
    w = _weights(D, H, K, rng)
    d = CacheDef(C=C, S=S, H=H, K=K, dtype=dtype, layout=layout, threshold=0.5, round_operands=(dtype == "bf16"),
                 predictor="fc_mlp")
    host = W.to_host_array(x)
    s0 = oracle.lookup(d, w, host)["score"]
    w["bs"] = float(np.float32(-np.median(s0)))
    ok = np.setdiff1d(np.arange(n), admit.inadmissible_rows(d, w, host)).astype(np.int32)
    assert len(ok) > n // 2
    want = oracle.lookup(d, w, host, row_index=ok)
    assert 0 < want["hit"].sum() < len(ok)
    cache = g.Cache(C, S, H, K, dtype, layout, 0.5, n, w, predictor="fc_mlp")
    assert cache.pool_variant == ("fc_flat" if D % 64 == 0 else "fc_flat_generic")
    m = len(ok)
    okd = torch.from_numpy(ok).cuda()
    xd = x.cuda()
    # the hidden layer alone (reported as the cache's features)
    feat = torch.full((m, H), -1.0, device="cuda")
    if H % 4 == 0 or D % 64 != 0:
        cache.pool(xd, okd, m, None, feat)
        torch.cuda.synchronize()
        tol = 2e-3 if dtype == "bf16" else 1e-4
        assert np.max(np.abs(feat.cpu().numpy() - want["pooled"])) <= tol
    out = {"pred_class": torch.zeros(m, dtype=torch.int32, device="cuda"), "confidence": torch.zeros(m, device="cuda"),
           "hit": torch.zeros(m, dtype=torch.uint8, device="cuda"), "logits": torch.zeros(m, K, device="cuda")}
    ids_out = torch.zeros(m, dtype=torch.int32, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    cache.lookup_compact(xd, okd, m, None, out["pred_class"], out["confidence"], out["hit"], out["logits"],
                         okd, ids_out, cnt)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    want_ideal = oracle.lookup(ideal_def(d), w, host, row_index=ok) if dtype == "bf16" else None
    # bf16 vs unrounded arithmetic: the rounding of W1 accumulates over D = C*S terms, so the gap
    # to the ideal result is wider than for the pooled predictors; the mirror bound is unchanged
    compare_lookup(got, want, want_ideal, dtype, f"fc_mlp {C}x{S}->{H}->{K}", tol_ideal=5e-2)
    want_ids = oracle.compact_misses(want["hit"], ok)
    assert int(cnt.item()) == len(want_ids)
    assert np.array_equal(ids_out.cpu().numpy()[:len(want_ids)], want_ids)
    # device-side count smaller than n_max; a second call gives identical bits
    n_dev = torch.tensor([m // 2], dtype=torch.int32, device="cuda")
    out2 = torch.full((m, K), -3.0, device="cuda")
    cache.lookup(xd, okd, m, n_dev, out["pred_class"], out["confidence"], out["hit"], out2)
    torch.cuda.synchronize()
    o2 = out2.cpu().numpy()
    assert np.array_equal(o2[:m // 2], got["logits"][:m // 2]) and np.all(o2[m // 2:] == -3.0)
    cache.close()
