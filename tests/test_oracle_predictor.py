"""Pins for the predictor (Section 3, table of predictor architectures:
Input -> Hidden Layer (ReLU) -FC-> Output) and the class distribution / argmax
(Section 3, "Training Learned Caches")."""
import math

import numpy as np
import torch

from oracle import CacheDef


def _w(W1, b1, W2, b2, ws=None, bs=0.0):
    W1, W2 = np.asarray(W1, np.float32), np.asarray(W2, np.float32)
    C, K = W1.shape[1], W2.shape[0]
    return {"W1": W1, "b1": np.asarray(b1, np.float32), "W2": W2, "b2": np.asarray(b2, np.float32),
            "ws": np.zeros(C + K, np.float32) if ws is None else np.asarray(ws, np.float32), "bs": bs}


def test_fc_hand_case(oracle):
    # small integers / halves: every product and sum is exact
    d = CacheDef(C=2, S=1, H=2, K=2)
    w = _w([[1, -1], [0.5, 2]], [0, -5], [[2, -7], [1, 3]], [0.25, 1])
    h = oracle.fc1_relu(d, w, np.array([2, 1], np.float32))
    assert h.tolist() == [1.0, 0.0]          # 2-1 = 1 ; 1+2-5 = -2 -> ReLU -> 0
    h = oracle.fc1_relu(d, w, np.array([0, 3], np.float32))
    assert h.tolist() == [0.0, 1.0]          # -3 -> 0 ; 0+6-5 = 1
    z = oracle.fc2(d, w, np.array([1.0, 0.0]))
    assert z.tolist() == [2.25, 2.0]
    z = oracle.fc2(d, w, np.array([0.0, 1.0]))
    assert z.tolist() == [-6.75, 4.0]


def test_fc_not_transposed(oracle):
    # W1[j,c] = 10 j + c, p = e_c  =>  h[j] = 10 j + c ; W2[k,j] = 10 k + j likewise
    C, H, K = 3, 4, 5
    W1 = (10 * np.arange(H)[:, None] + np.arange(C)[None, :]).astype(np.float32)
    W2 = (10 * np.arange(K)[:, None] + np.arange(H)[None, :]).astype(np.float32)
    d = CacheDef(C=C, S=1, H=H, K=K)
    w = _w(W1, np.zeros(H), W2, np.zeros(K))
    for c in range(C):
        e = np.zeros(C, np.float32); e[c] = 1
        assert oracle.fc1_relu(d, w, e).tolist() == [10.0 * j + c for j in range(H)]
    for j in range(H):
        e = np.zeros(H); e[j] = 1
        assert oracle.fc2(d, w, e).tolist() == [10.0 * k + j for k in range(K)]


def test_fc_zero_weights_and_identity(oracle):
    d = CacheDef(C=4, S=1, H=4, K=3)
    w = _w(np.zeros((4, 4)), [1, -1, 2, 0], np.zeros((3, 4)), [0.5, -0.5, 7])
    p = np.array([3, -1, 4, -1], np.float32)
    assert oracle.fc1_relu(d, w, p).tolist() == [1.0, 0.0, 2.0, 0.0]
    assert oracle.fc2(d, w, np.array([9.0, 9, 9, 9])).tolist() == [0.5, -0.5, 7.0]
    w = _w(np.eye(4), np.zeros(4), np.zeros((3, 4)), np.zeros(3))
    assert oracle.fc1_relu(d, w, p).tolist() == [3.0, 0.0, 4.0, 0.0]   # relu(p)


def test_fc_against_library_affine_map(oracle):
    g = np.random.default_rng(5)
    C, H, K = 37, 29, 11
    d = CacheDef(C=C, S=1, H=H, K=K)
    w = _w(g.standard_normal((H, C)), g.standard_normal(H), g.standard_normal((K, H)), g.standard_normal(K))
    p = g.standard_normal(C).astype(np.float32)
    h = oracle.fc1_relu(d, w, p)
    want_h = np.maximum(0.0, w["W1"].astype(np.float64) @ p.astype(np.float64) + w["b1"])
    assert np.allclose(h, want_h, rtol=0, atol=1e-12)
    z = oracle.fc2(d, w, h)
    want_z = torch.nn.functional.linear(torch.from_numpy(h), torch.from_numpy(w["W2"]).double(),
                                        torch.from_numpy(w["b2"]).double()).numpy()
    assert np.allclose(z, want_z, rtol=0, atol=1e-12)


def test_softmax_closed_forms(oracle):
    # K=2: q0 = logistic(z0 - z1); with z0 - z1 = ln 3 that is exactly 3/4
    q, cls = oracle.softmax_argmax(np.array([2.0 + math.log(3.0), 2.0]))
    assert abs(q[0] - 0.75) < 1e-15 and abs(q[1] - 0.25) < 1e-15 and cls == 0
    # constant logits: uniform, and the tie goes to the lowest index
    q, cls = oracle.softmax_argmax(np.full(7, -3.5))
    assert np.allclose(q, 1.0 / 7.0, atol=1e-16) and cls == 0
    # tie between two later maxima -> the earlier one
    q, cls = oracle.softmax_argmax(np.array([0.0, 5.0, 1.0, 5.0]))
    assert cls == 1
    # the largest entry last
    q, cls = oracle.softmax_argmax(np.array([0.0, 1.0, 2.0, 3.0]))
    assert cls == 3 and np.all(np.diff(q) > 0)


def test_softmax_invariants(oracle):
    g = np.random.default_rng(6)
    for K in (1, 2, 10, 1000):
        z = g.standard_normal(K) * 5
        q, cls = oracle.softmax_argmax(z)
        assert abs(q.sum() - 1.0) < 1e-12
        assert cls == int(np.argmax(z))
        q2, cls2 = oracle.softmax_argmax(z + 123.25)
        assert np.allclose(q, q2, rtol=1e-12, atol=0) and cls2 == cls
        want = torch.softmax(torch.from_numpy(z), dim=0).numpy()      # library third opinion
        assert np.allclose(q, want, rtol=1e-12, atol=1e-300)
    # large spread does not overflow
    q, cls = oracle.softmax_argmax(np.array([1000.0, 0.0, -1000.0]))
    assert q[0] == 1.0 and q[2] == 0.0 and cls == 0


def test_argmax_decided_in_fp32(oracle):
    # two logits that differ in fp64 but round to the same fp32: a tie, lowest index wins
    a = 1.0 + 2.0 ** -30
    q, cls = oracle.softmax_argmax(np.array([1.0, a]))
    assert cls == 0
