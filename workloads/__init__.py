"""Seeded synthetic inputs for the learned-cache lookup path.

This package only *draws inputs*: Zipf labels, per-class mean directions,
He-normal cache weights and ReLU-Gaussian / Gaussian activations with the
shapes of ResNet block outputs and BERT hidden states.  It holds none of the
lookup's arithmetic (no pooling, no FC, no softmax, no selector, no
compaction) and imports neither the CPU oracle nor the HIP library, so both
sides can be fed from it without sharing any of the method's code.
"""
from .spec import LayerSpec, WorkloadSpec, WORKLOADS, get_workload  # noqa: F401
from .synth import (  # noqa: F401
    zipf_labels,
    teacher_distribution,
    class_directions,
    cache_weights,
    activation_rows,
    activation_bulk,
    to_host_array,
)
