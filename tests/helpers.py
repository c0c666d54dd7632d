"""Shared plumbing of the GPU parity tests: build library caches and oracle inputs
from the same seeded workload, compare outputs to the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import workloads as W
from oracle import admit

# the benchmark spec tolerances: max abs error on logits and confidences
TOL = {"f32": 1e-4, "bf16": 2e-2}
# against the oracle run with the same bf16 operand rounding the deviation is much
# smaller: fp32 accumulation order plus the occasional one-ulp flip of a bf16 operand
TOL_MIRROR_BF16 = 5e-3


def make_cache(g, L, weights, max_rows):
    return g.Cache.from_layer(L, weights, max_rows)


def admissible_stack_inputs(spec: W.WorkloadSpec, calibrate_to=None):
    """Host tensors for every layer of a (small) workload with every (request, layer)
    pair admissible.  calibrate_to: per-layer hit rate to fit the selector bias to
    (on the oracle's scores), or None to keep the spec's biases."""
    from oracle.calibrate import bias_for_target
    K = spec.layers[0].K
    labels = W.zipf_labels(spec.batch, K, spec.zipf_s, spec.seed)
    defs = admit.cache_defs(spec, mirror=True)
    weights, acts = [], []
    req = np.arange(spec.batch)
    for l, (L, d) in enumerate(zip(spec.layers, defs)):
        w = W.cache_weights(spec, l)
        if calibrate_to is not None:
            raw = W.activation_rows(spec, l, labels, req)
            s0 = oracle.lookup(d, {**w, "bs": 0.0}, W.to_host_array(raw))["score"]
            w["bs"] = float(np.float32(bias_for_target(s0, L.threshold, calibrate_to)))
        act, _ = admit.admissible_layer(spec, l, labels, req, w)
        weights.append(w)
        acts.append(act)
    return labels, defs, weights, acts


def ideal_def(d):
    return oracle.CacheDef(**{**d.__dict__, "round_operands": False})


def compare_lookup(got: dict, want_mirror: dict, want_ideal, dtype: str, where="", tol_ideal=None):
    """got: numpy outputs of the library for n rows; want_*: oracle outputs.
    tol_ideal: tolerance against the unrounded arithmetic when it is not the default
    (the bf16-vs-unrounded gap grows with the length of the contraction)."""
    n = len(want_mirror["hit"])
    assert np.array_equal(got["pred_class"][:n], want_mirror["pred_class"]), f"{where}: class"
    assert np.array_equal(got["hit"][:n], want_mirror["hit"]), f"{where}: hit"
    tol = TOL[dtype]
    for ref, t in ((want_mirror, TOL_MIRROR_BF16 if dtype == "bf16" else tol), (want_ideal, tol_ideal or tol)):
        if ref is None:
            continue
        if got.get("logits") is not None:
            err = np.max(np.abs(got["logits"][:n].astype(np.float64) - ref["logits"])) if n else 0.0
            assert err <= t, f"{where}: logits max abs err {err} > {t}"
        err = np.max(np.abs(got["confidence"][:n].astype(np.float64) - ref["confidence"])) if n else 0.0
        assert err <= t, f"{where}: confidence max abs err {err} > {t}"


def to_device(act_host: torch.Tensor):
    return act_host.cuda()
