"""Pins for the oracle's pooling step (Section 3, pooling predictor: the spatial
size of the input is reduced before the projection; here a global mean)."""
import numpy as np
import torch

from oracle import CacheDef


def _d(C, S, dtype="f32", layout="ncs"):
    return CacheDef(C=C, S=S, H=1, K=1, dtype=dtype, layout=layout)


def test_hand_case(oracle):
    # two rows, C=2, S=3; means worked by hand: (1+2+3)/3=2, (-1+0+4)/3=1, 3, -3
    x = np.array([[[1, 2, 3], [-1, 0, 4]], [[3, 3, 3], [-3, -3, -3]]], np.float32)
    p = oracle.pool(_d(2, 3), x)
    assert p.tolist() == [[2.0, 1.0], [3.0, -3.0]]


def test_index_order_not_transposed(oracle):
    # x[r,c,s] = 100 r + 10 c + s: mean over s is 100 r + 10 c + (S-1)/2 exactly
    R, C, S = 3, 4, 5
    r, c, s = np.meshgrid(np.arange(R), np.arange(C), np.arange(S), indexing="ij")
    x = (100 * r + 10 * c + s).astype(np.float32)
    want = (100 * np.arange(R)[:, None] + 10 * np.arange(C)[None, :] + 2.0).astype(np.float32)
    assert np.array_equal(oracle.pool(_d(C, S), x), want)
    # the same values stored [n,S,C] give the same means
    xt = np.ascontiguousarray(x.transpose(0, 2, 1))
    assert np.array_equal(oracle.pool(_d(C, S, layout="nsc"), xt), want)


def test_constant_and_s1(oracle):
    x = np.full((2, 5, 7), 0.3, np.float32)
    assert np.all(oracle.pool(_d(5, 7), x) == np.float32(0.3))
    y = np.random.default_rng(0).standard_normal((4, 6, 1)).astype(np.float32)
    assert np.array_equal(oracle.pool(_d(6, 1), y), y[:, :, 0])


def test_sum_over_count_and_permutation(oracle):
    g = np.random.default_rng(1)
    x = g.standard_normal((3, 8, 49)).astype(np.float32)
    p = oracle.pool(_d(8, 49), x)
    exact = x.astype(np.float64).sum(axis=2) / 49.0           # library sum as third opinion
    assert np.array_equal(p, exact.astype(np.float32)) or np.max(np.abs(p - exact)) < 1e-7
    # pooled * count equals the sum (to fp32 rounding of p)
    assert np.allclose(p.astype(np.float64) * 49.0, x.astype(np.float64).sum(axis=2), rtol=1e-6, atol=1e-5)
    xp = x[:, :, g.permutation(49)]
    assert np.max(np.abs(oracle.pool(_d(8, 49), np.ascontiguousarray(xp)) - p)) <= 1e-7


def test_bf16_decode(oracle):
    t = torch.randn(2, 3, 16, generator=torch.Generator().manual_seed(3)).bfloat16()
    bits = t.view(torch.int16).numpy().view(np.uint16)
    want = (t.double().sum(dim=2) / 16.0).float().numpy()
    assert np.array_equal(oracle.pool(_d(3, 16, dtype="bf16"), bits), want)
    # exact special values: 1.0 = 0x3F80, -2.0 = 0xC000, 0.5 = 0x3F00
    bits = np.array([[[0x3F80, 0xC000, 0x3F00, 0x3F00]]], np.uint16)
    assert oracle.pool(_d(1, 4, dtype="bf16"), bits)[0, 0] == np.float32(0.0)


def test_row_selection(oracle):
    x = np.arange(4 * 2 * 3, dtype=np.float32).reshape(4, 2, 3)
    p = oracle.pool(_d(2, 3), x, rows=[3, 1])
    assert p.tolist() == [[19.0, 22.0], [7.0, 10.0]]
