"""Admissible synthetic rows.  TEST INFRASTRUCTURE ONLY (uses the oracle).

Class, hit flag and miss list are compared bit-exactly between the HIP library
and the oracle, which is only meaningful when no decision sits on a knife edge.
A (request, layer) pair is admissible when the top-2 logit gap and the distance
of the confidence from the threshold are both at least ``margin``; for bf16
caches this must hold, with the same class and hit decision, in both the
bf16-operand arithmetic and the unrounded arithmetic.  Inadmissible rows are
redrawn from their next per-row sub-seed.
"""
from __future__ import annotations

from typing import List

import numpy as np
import torch

import workloads as W
from . import CacheDef, lookup


def cache_defs(spec: W.WorkloadSpec, mirror: bool = True) -> List[CacheDef]:
    """Oracle-side description of every cache in a workload.  ``mirror`` selects the
    bf16-operand arithmetic for bf16 caches (the grading reference)."""
    return [CacheDef(C=L.C, S=L.S, H=L.H, K=L.K, dtype=L.dtype, layout=L.layout,
                     threshold=L.threshold, round_operands=(mirror and L.dtype == "bf16"),
                     predictor=L.predictor, in_hw=L.in_hw, out_hw=L.out_hw,
                     selector=L.selector, sel_hidden=L.sel_hidden, conv_ks=L.conv_ks)
            for L in spec.layers]


def _margins(out: dict, tau: float):
    z = np.sort(out["logits"].astype(np.float64), axis=1)
    gap = z[:, -1] - z[:, -2] if z.shape[1] > 1 else np.full(len(z), np.inf)
    return gap, np.abs(out["confidence"].astype(np.float64) - tau)


def inadmissible_rows(d_mirror: CacheDef, w: dict, act: np.ndarray, margin: float = 1e-3) -> np.ndarray:
    outs = [lookup(d_mirror, w, act)]
    if d_mirror.round_operands:
        d_ideal = CacheDef(**{**d_mirror.__dict__, "round_operands": False})
        outs.append(lookup(d_ideal, w, act))
    bad = np.zeros(len(outs[0]["hit"]), bool)
    for o in outs:
        gap, dist = _margins(o, d_mirror.threshold)
        bad |= (gap < margin) | (dist < margin)
    if len(outs) == 2:
        bad |= outs[0]["pred_class"] != outs[1]["pred_class"]
        bad |= outs[0]["hit"] != outs[1]["hit"]
    return np.nonzero(bad)[0]


def admissible_layer(spec: W.WorkloadSpec, layer: int, labels: np.ndarray, requests,
                     weights: dict, margin: float = 1e-3, max_attempts: int = 20):
    """Host activations [len(requests), ...] for one layer with every row admissible.
    Returns (tensor, attempts_used_per_row)."""
    requests = np.asarray(requests, np.int64)
    d = cache_defs(spec)[layer]
    attempts = np.zeros(len(requests), np.int64)
    act = W.activation_rows(spec, layer, labels, requests, attempts, device="cpu")
    for _ in range(max_attempts):
        bad = inadmissible_rows(d, weights, W.to_host_array(act), margin)
        if len(bad) == 0:
            return act, attempts
        attempts[bad] += 1
        act[torch.from_numpy(bad)] = W.activation_rows(spec, layer, labels, requests[bad],
                                                       attempts[bad], device="cpu")
    raise RuntimeError(f"layer {layer}: rows still inadmissible after {max_attempts} redraws")
