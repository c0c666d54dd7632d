"""Fit the per-layer selector biases of the hit-rate-controlled workloads.

TEST INFRASTRUCTURE (uses the oracle).  Writes ``workloads/calibration.json``:

    python -m oracle.calibrate [--sample N] [--device cpu|cuda] [--threads T] [--out FILE] [workload ...]

The stored file was written on an MI355X machine with ``--sample 4096 --device cuda`` for the workloads of the
five configs and their selector / pooling / convolution variants (so the tensors scored are bit for bit
the ones the benchmark times), and with a CPU-drawn sample for resnet50_fc, whose oracle needs about a
second per lookup.

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


def _scores(d, w, act, rows, threads):
    """Zero-bias oracle scores of the given rows of act, row shards on several host threads (each call
    is the single-threaded oracle; the C library runs outside the interpreter lock)."""
    from concurrent.futures import ThreadPoolExecutor
    rows = np.ascontiguousarray(rows, np.int32)
    shards = [s for s in np.array_split(rows, max(1, min(threads, len(rows)))) if len(s)]
    with ThreadPoolExecutor(len(shards)) as ex:
        outs = list(ex.map(lambda s: lookup(d, w, act, row_index=s, n=len(s))["score"], shards))
    return np.concatenate(outs)


def calibrate(name: str, sample: int = 512, verbose: bool = True, device: str = "cpu", threads: int = 1) -> dict:
    """sample >= batch: every layer's tensor is drawn exactly as the benchmark and the full-batch GPU tests
    draw it -- the whole batch from the layer's one stream on `device` ("gather" storage), or the rows
    still active ("dense" storage) -- so on the same device the biases are fitted on the very tensors
    that are later timed and the hit-rate ramp holds by construction.  A smaller sample draws only its
    own rows (a statistical fit, for predictors whose oracle is too slow for the whole batch)."""
    spec = _build()[name]          # the uncalibrated spec: bs = 0 everywhere
    targets = HIT_TARGETS[name]
    K = spec.layers[0].K
    labels = W.zipf_labels(spec.batch, K, spec.zipf_s, spec.seed)
    whole = sample >= spec.batch
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
        if whole and spec.storage == "gather":
            act = W.to_host_array(W.activation_bulk(spec, l, labels, np.arange(spec.batch), device=device))
            score = _scores(d, w, act, active, threads)
        else:
            act = W.to_host_array(W.activation_bulk(spec, l, labels, active, device=device))
            score = _scores(d, w, act, np.arange(len(active)), threads)
        del act
        b = bias_for_target(score, L.threshold, targets[l])
        b = float(np.float32(b))
        hit = (score + b) > math.log(L.threshold / (1.0 - L.threshold))
        bs.append(b)
        achieved.append(float(hit.mean()))
        if verbose:
            print(f"{name} layer {l:2d}: n={len(active):4d} target={targets[l]:.3f} "
                  f"hit={hit.mean():.3f} bs={b:+.4f}  ({time.time() - t0:.1f}s)", flush=True)
        active = active[~hit]
    return {"bs": bs, "target_hit": [float(t) for t in targets], "sample_hit": achieved,
            "sample_requests": int(min(sample, spec.batch)), "drawn_on": device,
            "cumulative_sample_hit": 1.0 - len(active) / float(min(sample, spec.batch))}


def main(argv):
    """python -m oracle.calibrate [--sample N] [--device cpu|cuda] [--threads T] [--out FILE] [workload ...]"""
    opts = {"--sample": "512", "--device": "cpu", "--threads": "1", "--out": _OUT}
    for key in list(opts):
        if key in argv:
            i = argv.index(key)
            opts[key] = argv[i + 1]
            argv = argv[:i] + argv[i + 2:]
    names = argv or sorted(HIT_TARGETS)
    cal = {}
    if os.path.exists(_OUT):
        with open(_OUT) as f:
            cal = json.load(f)
    for n in names:
        cal[n] = calibrate(n, sample=int(opts["--sample"]), device=opts["--device"], threads=int(opts["--threads"]))
        with open(opts["--out"], "w") as f:
            json.dump(cal, f, indent=1)
            f.write("\n")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
