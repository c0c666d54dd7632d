"""Pins for the bf16 cache arithmetic of the oracle: the operands of the two FC
layers (weights, pooled features, hidden activations) are bf16 values, products
and sums are exact/fp64.  The paper states no precision; bf16 is this build's
reading for the bf16 workloads."""
import numpy as np
import torch

from oracle import CacheDef


def test_round_hand_cases(oracle):
    r = oracle.round_bf16
    assert r(1.0) == 1.0
    assert r(1.0 + 2.0 ** -8) == 1.0                       # tie -> even mantissa
    assert r(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6       # tie -> even mantissa (up)
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert r(-0.1) == -0.10009765625
    assert r(0.0) == 0.0
    assert r(255.0) == 255.0 and r(257.0) == 256.0 and r(259.0) == 260.0
    assert r(2.0 ** -133) == 2.0 ** -133 and r(2.0 ** -135) == 0.0   # subnormal spacing


def test_round_matches_library_conversion_on_fp32_inputs(oracle):
    g = torch.Generator().manual_seed(0)
    x = torch.randn(20000, generator=g) * torch.logspace(-30, 30, 20000)
    want = x.bfloat16().double().numpy()
    got = np.array([oracle.round_bf16(float(v)) for v in x.double()])
    assert np.array_equal(got, want)


def test_rounded_lookup_against_library_ops(oracle):
    g = np.random.default_rng(2)
    n, C, S, H, K = 5, 24, 10, 16, 12
    x = torch.from_numpy(g.standard_normal((n, C, S)).astype(np.float32)).bfloat16()
    bits = x.view(torch.int16).numpy().view(np.uint16)
    w = {"W1": (g.standard_normal((H, C)) * 0.3).astype(np.float32), "b1": (g.standard_normal(H) * 0.1).astype(np.float32),
         "W2": (g.standard_normal((K, H)) * 0.3).astype(np.float32), "b2": (g.standard_normal(K) * 0.1).astype(np.float32),
         "ws": (g.standard_normal(C + K) * 0.5).astype(np.float32), "bs": -0.1}
    d = CacheDef(C=C, S=S, H=H, K=K, dtype="bf16", threshold=0.5, round_operands=True)
    out = oracle.lookup(d, w, bits)
    bf = lambda t: t.float().bfloat16().double()
    p32 = x.double().mean(dim=2).float()
    assert np.array_equal(out["pooled"], p32.numpy())
    W1, W2 = bf(torch.from_numpy(w["W1"])), bf(torch.from_numpy(w["W2"]))
    h = torch.relu(bf(p32) @ W1.T + torch.from_numpy(w["b1"]).double())
    # h is rounded from fp64 straight to bf16; going through fp32 first can differ
    # only on double-rounding ties, which do not occur for these values
    z = bf(h) @ W2.T + torch.from_numpy(w["b2"]).double()
    assert np.allclose(out["logits"], z.numpy(), rtol=0, atol=1e-6)
    q = torch.softmax(z, dim=1)
    u = torch.cat([p32.double(), q], dim=1) @ torch.from_numpy(w["ws"]).double() + float(np.float32(-0.1))
    assert np.allclose(out["score"], u.numpy(), rtol=0, atol=1e-12)
    # the unrounded arithmetic gives different, nearby logits
    d0 = CacheDef(C=C, S=S, H=H, K=K, dtype="bf16", threshold=0.5, round_operands=False)
    out0 = oracle.lookup(d0, w, bits)
    diff = np.max(np.abs(out0["logits"] - out["logits"]))
    assert 0 < diff < 2e-2
