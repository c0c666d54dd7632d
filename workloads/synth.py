"""Seeded draws: labels, class directions, cache weights, activations.

Small objects (labels, directions, weights) come from numpy PCG64
streams keyed by ``SeedSequence`` on the host, so they are the same bits on
every machine.  Bulk activation noise comes from ``torch.randn`` on whichever
device the caller names (host for the oracle-only work, GPU for the big
timed tensors); the resulting tensor is the single source both the oracle and
the HIP library read, so they always see identical bits.
"""
from __future__ import annotations

import numpy as np
import torch

from .spec import LayerSpec, WorkloadSpec

_TAG_LABELS, _TAG_DIRS, _TAG_WEIGHTS, _TAG_ROW, _TAG_BULK, _TAG_SELECTOR, _TAG_TEACHER = 1, 2, 3, 4, 5, 6, 7


def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, *key])))


def _torch_seed(seed: int, *key: int) -> int:
    ss = np.random.SeedSequence([seed, *key])
    return int(ss.generate_state(1, dtype=np.uint64)[0] >> np.uint64(1))


def zipf_labels(batch: int, K: int, s: float, seed: int) -> np.ndarray:
    """Labels with P(class k) proportional to (k+1)^-s, by inverse CDF of a seeded uniform."""
    ranks = np.arange(1, K + 1, dtype=np.float64)
    pmf = ranks ** (-float(s))
    cdf = np.cumsum(pmf / pmf.sum())
    cdf[-1] = 1.0
    u = _rng(seed, _TAG_LABELS).random(batch)
    return np.searchsorted(cdf, u, side="right").astype(np.int32).clip(0, K - 1)


def teacher_distribution(labels: np.ndarray, K: int, seed: int, accuracy: float = 0.9,
                         peak: float = 0.8) -> np.ndarray:
    """[n, K] float32 rows on the simplex standing in for the base DNN's output on requests whose
    true classes are `labels`: mass `peak` on the base model's answer (the true class with
    probability `accuracy`, else another class drawn uniformly), the rest spread by a seeded
    Dirichlet draw."""
    n = len(labels)
    rng = _rng(seed, _TAG_TEACHER)
    wrong = rng.random(n) >= accuracy
    other = (np.asarray(labels) + 1 + rng.integers(0, max(K - 1, 1), n)) % K
    answer = np.where(wrong, other, labels)
    Y = rng.dirichlet(np.full(K, 0.3), size=n) * (1.0 - peak)
    Y[np.arange(n), answer] += peak
    Y = Y.astype(np.float32)
    return Y / Y.sum(axis=1, keepdims=True, dtype=np.float32)


def class_directions(spec: WorkloadSpec, layer: int) -> np.ndarray:
    """[K, C] float32: one unit-norm direction per class for this layer."""
    L = spec.layers[layer]
    d = _rng(spec.seed, _TAG_DIRS, layer).standard_normal((L.K, L.C))
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    return d.astype(np.float32)


def cache_weights(spec: WorkloadSpec, layer: int) -> dict:
    """He-normal fp32 weights N(0, 2/fan_in); zero predictor biases; selector bias from the spec.

    Shapes follow the [out, in] convention: W1 [H,C], W2 [K,H], ws [C+K] with the
    pooled features first and the class probabilities after them.
    """
    w = _predictor_and_linear_selector(spec, layer)
    L = spec.layers[layer]
    if L.selector == "hidden":
        # drawn from a stream of its own so the predictor weights equal those of the linear-selector stack
        g = _rng(spec.seed, _TAG_SELECTOR, layer)
        n_in = L.F + L.K
        w["Ws"] = (g.standard_normal((L.sel_hidden, n_in)) * np.sqrt(2.0 / n_in)).astype(np.float32)
        w["cs"] = np.zeros(L.sel_hidden, np.float32)
        w["vs"] = (g.standard_normal(L.sel_hidden) * np.sqrt(2.0 / L.sel_hidden)).astype(np.float32)
    return w


def _predictor_and_linear_selector(spec: WorkloadSpec, layer: int) -> dict:
    L = spec.layers[layer]
    g = _rng(spec.seed, _TAG_WEIGHTS, layer)
    if L.predictor == "pool_fc":
        # Pool(h): no hidden FC; the output FC reads the F pooled features
        W2 = (g.standard_normal((L.K, L.F)) * np.sqrt(2.0 / L.F)).astype(np.float32)
        ws = (g.standard_normal(L.F + L.K) * np.sqrt(2.0 / (L.F + L.K))).astype(np.float32)
        return {"W1": None, "b1": None, "W2": W2, "b2": np.zeros(L.K, np.float32), "ws": ws, "bs": float(L.bs)}
    if L.predictor == "conv_fc":
        # Conv(k,s): H filters [H, C, k, k] (fan-in C*k*k), then the output FC over the F hidden values
        k = L.conv_ks[0]
        W1 = (g.standard_normal((L.H, L.C, k, k)) * np.sqrt(2.0 / (L.C * k * k))).astype(np.float32)
        W2 = (g.standard_normal((L.K, L.F)) * np.sqrt(2.0 / L.F)).astype(np.float32)
        ws = (g.standard_normal(L.F + L.K) * np.sqrt(2.0 / (L.F + L.K))).astype(np.float32)
        return {"W1": W1, "b1": np.zeros(L.H, np.float32), "W2": W2, "b2": np.zeros(L.K, np.float32),
                "ws": ws, "bs": float(L.bs)}
    if L.predictor == "fc_mlp":
        # FC(h): the first FC reads the whole flattened row (D = C*S inputs); drawn in float32
        # row blocks to keep the host footprint at one copy of the matrix
        D = L.C * L.S
        W1 = np.empty((L.H, D), np.float32)
        scale = np.float32(np.sqrt(2.0 / D))
        for j0 in range(0, L.H, 64):
            W1[j0:j0 + 64] = g.standard_normal((min(64, L.H - j0), D), dtype=np.float32) * scale
        W2 = (g.standard_normal((L.K, L.H)) * np.sqrt(2.0 / L.H)).astype(np.float32)
        ws = (g.standard_normal(L.H + L.K) * np.sqrt(2.0 / (L.H + L.K))).astype(np.float32)
        return {"W1": W1, "b1": np.zeros(L.H, np.float32), "W2": W2, "b2": np.zeros(L.K, np.float32),
                "ws": ws, "bs": float(L.bs)}
    W1 = (g.standard_normal((L.H, L.C)) * np.sqrt(2.0 / L.C)).astype(np.float32)
    W2 = (g.standard_normal((L.K, L.H)) * np.sqrt(2.0 / L.H)).astype(np.float32)
    ws = (g.standard_normal(L.C + L.K) * np.sqrt(2.0 / (L.C + L.K))).astype(np.float32)
    return {
        "W1": W1, "b1": np.zeros(L.H, np.float32),
        "W2": W2, "b2": np.zeros(L.K, np.float32),
        "ws": ws, "bs": float(L.bs),
    }


def _torch_dtype(L: LayerSpec):
    return torch.float32 if L.dtype == "f32" else torch.bfloat16


def _shape(L: LayerSpec, n: int):
    return (n, L.C, L.S) if L.layout == "ncs" else (n, L.S, L.C)


def _fill(L: LayerSpec, out: torch.Tensor, mean_rows: torch.Tensor, gen: torch.Generator):
    """out[i] = cast(relu?(N(0,1) + mean_rows[i][c]))."""
    n = out.shape[0]
    noise = torch.randn(_shape(L, n), generator=gen, device=out.device, dtype=torch.float32)
    if L.layout == "ncs":
        noise += mean_rows.view(n, L.C, 1)
    else:
        noise += mean_rows.view(n, 1, L.C)
    if L.relu:
        noise.clamp_(min=0.0)
    out.copy_(noise)


def activation_rows(spec: WorkloadSpec, layer: int, labels: np.ndarray, requests,
                    attempts=None, device="cpu") -> torch.Tensor:
    """Activations of the given requests at one layer, one seeded stream per
    (layer, request, attempt), so that a single request can be redrawn alone.

    Returns a tensor of shape [len(requests), C, S] (ncs) or [len(requests), S, C] (nsc).
    """
    L = spec.layers[layer]
    requests = np.asarray(requests, dtype=np.int64)
    attempts = np.zeros(len(requests), np.int64) if attempts is None else np.asarray(attempts)
    dirs = torch.from_numpy(class_directions(spec, layer)).to(device)
    out = torch.empty(_shape(L, len(requests)), dtype=_torch_dtype(L), device=device)
    gen = torch.Generator(device=device)
    for j, (r, a) in enumerate(zip(requests, attempts)):
        gen.manual_seed(_torch_seed(spec.seed, _TAG_ROW, layer, int(r), int(a)))
        mean = (L.gamma * dirs[int(labels[int(r)])]).view(1, L.C)
        _fill(L, out[j:j + 1], mean, gen)
    return out


def activation_bulk(spec: WorkloadSpec, layer: int, labels: np.ndarray, requests,
                    device="cuda", chunk_bytes: int = 1 << 30) -> torch.Tensor:
    """Activations of many requests at one layer from one seeded stream (fast path
    for the large timed tensors).  Row j holds request ``requests[j]``."""
    L = spec.layers[layer]
    requests = np.asarray(requests, dtype=np.int64)
    n = len(requests)
    dirs = torch.from_numpy(class_directions(spec, layer)).to(device)
    lab = torch.from_numpy(np.asarray(labels)[requests].astype(np.int64)).to(device)
    out = torch.empty(_shape(L, n), dtype=_torch_dtype(L), device=device)
    gen = torch.Generator(device=device)
    gen.manual_seed(_torch_seed(spec.seed, _TAG_BULK, layer, n))
    rows_per_chunk = max(1, chunk_bytes // (L.C * L.S * 4))
    for lo in range(0, n, rows_per_chunk):
        hi = min(n, lo + rows_per_chunk)
        mean = L.gamma * dirs[lab[lo:hi]]
        _fill(L, out[lo:hi], mean, gen)
    return out


def to_host_array(t: torch.Tensor) -> np.ndarray:
    """Host numpy view of an activation tensor: float32 as is, bf16 as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
