"""Fit the per-layer selector biases of the hit-rate-controlled workloads.

TEST INFRASTRUCTURE (uses the oracle).  Writes ``workloads/calibration.json``:

    python -m oracle.calibrate [--sample N] [workload ...]

The configs ask for a hit rate that rises with depth (the paper's per-block
tables show exactly that shape).  With random weights the selector score is
close to a per-class constant, so a target rate is met by shifting the selector
bias: for each layer, in stack order, the oracle scores the requests still
active with bias 0, and the bias is set so that the wanted fraction of them
clears the threshold.  Only seeded generators and the oracle are involved; the
HIP library is never consulted.
"""
from __future__ import annotations

import json
import math
import os
import sys
import time

import numpy as np

import workloads as W
from workloads.spec import HIT_TARGETS, _build
from . import lookup
from .admit import cache_defs

_OUT = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "workloads", "calibration.json")


def bias_for_target(score0: np.ndarray, tau: float, target: float) -> float:
    """Bias that makes round(target*n) of the given zero-bias scores exceed logit(tau),
    placed midway between the last hit and the first miss."""
    n = len(score0)
    cut = math.log(tau / (1.0 - tau))
    k = int(round(target * n))
    s = np.sort(score0)[::-1]
    if n == 0:
        return 0.0
    if k <= 0:
        return cut - (s[0] + 1.0)
    if k >= n:
        return cut - (s[-1] - 1.0)
    return cut - 0.5 * (s[k - 1] + s[k])


def calibrate(name: str, sample: int = 512, verbose: bool = True) -> dict:
    spec = _build()[name]          # the uncalibrated spec: bs = 0 everywhere
    targets = HIT_TARGETS[name]
    K = spec.layers[0].K
    labels = W.zipf_labels(spec.batch, K, spec.zipf_s, spec.seed)
    active = np.arange(min(sample, spec.batch), dtype=np.int64)
    defs = cache_defs(spec, mirror=True)
    bs, achieved = [], []
    for l, (L, d) in enumerate(zip(spec.layers, defs)):
        if len(active) == 0:
            bs.append(0.0)
            achieved.append(None)
            continue
        t0 = time.time()
        w = W.cache_weights(spec, l)
        act = W.to_host_array(W.activation_bulk(spec, l, labels, active, device="cpu"))
        out = lookup(d, w, act)
        b = bias_for_target(out["score"], L.threshold, targets[l])
        hit = (out["score"] + b) > math.log(L.threshold / (1.0 - L.threshold))
        bs.append(float(np.float32(b)))
        achieved.append(float(hit.mean()))
        if verbose:
            print(f"{name} layer {l:2d}: n={len(active):4d} target={targets[l]:.3f} "
                  f"hit={hit.mean():.3f} bs={b:+.4f}  ({time.time() - t0:.1f}s)", flush=True)
        active = active[~hit]
    return {"bs": bs, "target_hit": [float(t) for t in targets], "sample_hit": achieved,
            "sample_requests": int(min(sample, spec.batch)),
            "cumulative_sample_hit": 1.0 - len(active) / float(min(sample, spec.batch))}


def main(argv):
    sample = 512
    if "--sample" in argv:
        i = argv.index("--sample")
        sample = int(argv[i + 1])
        argv = argv[:i] + argv[i + 2:]
    names = argv or sorted(HIT_TARGETS)
    cal = {}
    if os.path.exists(_OUT):
        with open(_OUT) as f:
            cal = json.load(f)
    for n in names:
        cal[n] = calibrate(n, sample=sample)
        with open(_OUT, "w") as f:
            json.dump(cal, f, indent=1)
            f.write("\n")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
