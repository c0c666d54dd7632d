"""Shapes of the five synthetic workloads.

Each workload is a stack of learned caches, one per hooked block of a base
network (the paper places a lookup after every layer, Section 2 "caching
proposal" figure and Section 3).  Only shapes, dtypes and the knobs of the
input distribution live here.
"""
from __future__ import annotations

import json
import os
from dataclasses import dataclass, field, replace
from typing import List, Optional


@dataclass(frozen=True)
class LayerSpec:
    C: int            # channels / hidden width of the activation
    S: int            # reduced length: H*W of the feature map, or tokens
    H: int            # predictor hidden width
    K: int            # classes
    layout: str       # "ncs" ([n,C,S], S contiguous) or "nsc" ([n,S,C], C contiguous)
    dtype: str        # "f32" or "bf16"
    threshold: float  # selector threshold tau
    gamma: float      # class-mean scale: element mean = gamma * d[label][c]
    relu: bool        # ReLU-Gaussian (CNN block outputs) or plain Gaussian (tokens)
    bs: float = 0.0   # selector bias (calibrated per layer for the hit-rate ramps)
    target_hit: Optional[float] = None  # per-layer hit-rate target the bias was fitted to
    predictor: str = "gap_mlp"   # "gap_mlp" | "pool_fc" (the paper's Pool(h): adaptive pool -> ReLU -> FC)
                                 # | "fc_mlp" (the paper's FC(h): flattened activation -> FC -> ReLU -> FC)
    in_hw: tuple = (0, 0)        # pool_fc: feature-map size, S = in_h*in_w
    out_hw: tuple = (0, 0)       # pool_fc: pooled map; F = C*out_h*out_w features
    selector: str = "linear"     # "linear" | "softmax" | "hidden" (selector network with one hidden layer)
    sel_hidden: int = 0          # units of that hidden layer
    conv_ks: tuple = (0, 0)      # conv_fc (the paper's Conv(k,s)): filter size and stride; H filters, map in_hw

    @property
    def F(self) -> int:
        """Features the pooling step hands to the FC layers."""
        if self.predictor == "pool_fc":
            return self.C * self.out_hw[0] * self.out_hw[1]
        if self.predictor == "conv_fc":
            k, s = self.conv_ks
            return self.H * ((self.in_hw[0] - k) // s + 1) * ((self.in_hw[1] - k) // s + 1)
        return self.H if self.predictor == "fc_mlp" else self.C

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def row_bytes(self) -> int:
        return self.C * self.S * self.elem_bytes


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    batch: int
    zipf_s: float
    seed: int
    layers: List[LayerSpec] = field(default_factory=list)
    # "gather": every layer holds the full batch, lookups index it by request id.
    # "dense":  layer l holds only the rows still active, in miss-list order.
    storage: str = "gather"

    def scaled(self, batch: int, name: Optional[str] = None) -> "WorkloadSpec":
        """Same stack at another batch size (parity-test sized variants)."""
        return replace(self, batch=batch, name=name or f"{self.name}@{batch}")


def _resnet_stack(blocks, H, K, dtype, tau, gammas, pool_out=None):
    """pool_out: None for the global-pool predictor, else {hw: pooled side} for Pool(h)."""
    layers = []
    idx = 0
    total = sum(b for _, _, b in blocks)
    for (C, hw, reps) in blocks:
        for _ in range(reps):
            g = gammas[0] + (gammas[1] - gammas[0]) * (idx / max(1, total - 1))
            extra = {}
            if pool_out is not None:
                extra = dict(predictor="pool_fc", in_hw=(hw, hw), out_hw=(pool_out[hw], pool_out[hw]))
            layers.append(LayerSpec(C=C, S=hw * hw, H=0 if pool_out is not None else H, K=K, layout="ncs",
                                    dtype=dtype, threshold=tau, gamma=g, relu=True, **extra))
            idx += 1
    return layers


def _linear_ramp(first, last, n):
    return [first + (last - first) * i / max(1, n - 1) for i in range(n)]


def _build():
    w = {}
    # cfg 0: one tiny fp32 cache, [64,64,8,8], 64 -> 128 -> 10, selector 74 -> 1, tau 0.5
    w["tiny"] = WorkloadSpec(
        name="tiny", batch=64, zipf_s=1.1, seed=0,
        layers=[LayerSpec(C=64, S=64, H=128, K=10, layout="ncs", dtype="f32",
                          threshold=0.5, gamma=6.0, relu=True)])
    # cfg 1: ResNet-18-shaped, 8 basic-block outputs, fp32, batch 256, tau 0.6
    w["resnet18"] = WorkloadSpec(
        name="resnet18", batch=256, zipf_s=1.1, seed=0,
        layers=_resnet_stack([(64, 56, 2), (128, 28, 2), (256, 14, 2), (512, 7, 2)],
                             H=256, K=1000, dtype="f32", tau=0.6, gammas=(8.0, 24.0)))
    # cfg 2: ResNet-50-shaped, 16 bottleneck outputs (3+4+6+3), bf16, batch 512
    w["resnet50"] = WorkloadSpec(
        name="resnet50", batch=512, zipf_s=1.1, seed=0,
        layers=_resnet_stack([(256, 56, 3), (512, 28, 4), (1024, 14, 6), (2048, 7, 3)],
                             H=512, K=1000, dtype="bf16", tau=0.6, gammas=(8.0, 32.0)))
    # cfg 3: BERT-base-shaped, 12 encoder outputs [1024,128,768], token-mean pool
    w["bert_base"] = WorkloadSpec(
        name="bert_base", batch=1024, zipf_s=1.2, seed=0,
        layers=[LayerSpec(C=768, S=128, H=256, K=20, layout="nsc", dtype="bf16",
                          threshold=0.5, gamma=4.0 + 1.0 * i, relu=False)
                for i in range(12)])
    # cfg 4: ResNet-152-shaped, 50 block outputs (3+8+36+3), bf16, streaming batch 4096,
    # each layer stored only for the rows still active
    w["resnet152"] = WorkloadSpec(
        name="resnet152", batch=4096, zipf_s=1.1, seed=0, storage="dense",
        layers=_resnet_stack([(256, 56, 3), (512, 28, 8), (1024, 14, 36), (2048, 7, 3)],
                             H=512, K=1000, dtype="bf16", tau=0.6, gammas=(8.0, 32.0)))
    # The paper's own Pool(h) variant on the ResNet-50 shapes: pooled maps chosen so that
    # h = C*s*s is the paper's 4096 / 8192 (Section 7 "Default Parameters")
    w["resnet50_pool"] = WorkloadSpec(
        name="resnet50_pool", batch=512, zipf_s=1.1, seed=0,
        layers=_resnet_stack([(256, 56, 3), (512, 28, 4), (1024, 14, 6), (2048, 7, 3)],
                             H=0, K=1000, dtype="bf16", tau=0.6, gammas=(8.0, 32.0),
                             pool_out={56: 4, 28: 4, 14: 2, 7: 2}))
    # The paper's FC(h) variant (h = 1024, its default) at six ResNet-50 blocks -- the paper's GPU
    # composition for ResNet-50 ends up with six FC caches (Section 7.1).  Blocks 3, 6, 9, 11, 13, 16.
    fc_blocks = [(256, 56), (512, 28), (1024, 14), (1024, 14), (1024, 14), (2048, 7)]
    w["resnet50_fc"] = WorkloadSpec(
        name="resnet50_fc", batch=512, zipf_s=1.1, seed=0,
        layers=[LayerSpec(C=C, S=hw * hw, H=1024, K=1000, layout="ncs", dtype="bf16", threshold=0.6,
                          gamma=8.0 + 4.8 * i, relu=True, predictor="fc_mlp")
                for i, (C, hw) in enumerate(fc_blocks)])
    # The paper's Conv(k,s) variant on the ResNet-50 shapes, 8 filters: Conv(5,2) on the 56x56 and 28x28
    # maps, Conv(3,1) on the 14x14 and 7x7 ones (the two settings of Section 7 "Default Parameters"),
    # i.e. 5408 / 1152 / 1152 / 200 hidden values
    conv_layers = []
    for l in w["resnet50"].layers:
        hw = int(round(l.S ** 0.5))
        conv_layers.append(replace(l, H=8, predictor="conv_fc", in_hw=(hw, hw), conv_ks=(5, 2) if hw >= 28 else (3, 1)))
    w["resnet50_conv"] = replace(w["resnet50"], name="resnet50_conv", layers=conv_layers)
    # The resnet50 stack with the paper's selector shape: one hidden layer (Section 3, "Selector
    # Network Design") of 64 units over [pooled ; class probabilities]
    w["resnet50_hsel"] = replace(w["resnet50"], name="resnet50_hsel",
                                 layers=[replace(l, selector="hidden", sel_hidden=64) for l in w["resnet50"].layers])
    return w


# Per-layer hit-rate targets (fraction of the rows looked up at that layer).
# resnet50: linear ramp whose product of miss rates leaves ~40 % after layer 16.
# resnet152: 2 % -> 70 % linear ramp over the 50 layers.
HIT_TARGETS = {
    # resnet18 / bert_base: the configs leave the rate open; with random weights the
    # un-tuned rate is degenerate (all or nothing), so a ramp in the shape of the paper's
    # per-block hit-rate table is used: ~84 % and ~75 % cumulative by the last layer.
    "resnet18": _linear_ramp(0.05, 0.35, 8),
    "resnet50": [0.0065 * (i + 1) for i in range(16)],
    "resnet50_pool": [0.0065 * (i + 1) for i in range(16)],
    "resnet50_hsel": [0.0065 * (i + 1) for i in range(16)],
    "resnet50_conv": [0.0065 * (i + 1) for i in range(16)],
    "resnet50_fc": _linear_ramp(0.05, 0.20, 6),
    "bert_base": _linear_ramp(0.02, 0.20, 12),
    "resnet152": _linear_ramp(0.02, 0.70, 50),
}

_CAL_PATH = os.path.join(os.path.dirname(__file__), "calibration.json")


def _apply_calibration(w):
    """Fold the fitted selector biases (a stored text fixture) into the specs."""
    if not os.path.exists(_CAL_PATH):
        return w
    with open(_CAL_PATH) as f:
        cal = json.load(f)
    for name, entry in cal.items():
        if name not in w:
            continue
        bs = entry["bs"]
        tgt = entry.get("target_hit", [None] * len(bs))
        spec = w[name]
        if len(bs) != len(spec.layers):
            continue
        layers = [replace(l, bs=float(b), target_hit=t) for l, b, t in zip(spec.layers, bs, tgt)]
        w[name] = replace(spec, layers=layers)
    return w


WORKLOADS = _apply_calibration(_build())


def get_workload(name: str) -> WorkloadSpec:
    if name not in WORKLOADS:
        raise KeyError(f"unknown workload {name!r}; have {sorted(WORKLOADS)}")
    return WORKLOADS[name]
