"""A whole stack pass captured into a HIP graph replays to the eager result (the library
allocates nothing and never synchronises inside a call, so its launches can be captured)."""
import numpy as np
import pytest
import torch

import paper_2101_07344_amd as g
import workloads as W

pytestmark = pytest.mark.gpu


def _snapshot(stack, n_layers):
    return ([t.clone() for t in stack.hit], [t.clone() for t in stack.pred_class],
            [t.clone() for t in stack.confidence], [t.clone() for t in stack.ids], stack.counts.clone())


def _same(a, b):
    """Equal counts, and equal outputs on the valid prefix of every layer (entries past the
    active count are left untouched by the library)."""
    if not torch.equal(a[4], b[4]):
        return False
    counts = a[4].tolist()
    for l in range(len(a[0])):
        n = counts[l]
        if not all(torch.equal(a[k][l][:n], b[k][l][:n]) for k in range(3)):
            return False
    return all(torch.equal(a[3][l][:counts[l]], b[3][l][:counts[l]]) for l in range(len(a[3])))


@pytest.mark.parametrize("name,batch,layers", [
    ("resnet18", 48, slice(0, 6)), ("bert_base", 96, slice(0, 6)),
    # the predictor / selector variants: Pool(h), Conv(k,s) incl. its split + reduce kernels, hidden-layer selector
    ("resnet50_pool", 40, slice(5, 9)), ("resnet50_conv", 24, slice(5, 9)), ("resnet50_hsel", 40, slice(5, 9)),
])
def test_graph_replay_equals_eager(name, batch, layers):
    base = W.get_workload(name)
    spec = W.WorkloadSpec(name=f"{name}@{batch}", batch=batch, zipf_s=base.zipf_s, seed=base.seed,
                          layers=base.layers[layers], storage="gather")
    labels = W.zipf_labels(batch, spec.layers[0].K, spec.zipf_s, spec.seed)
    weights = [W.cache_weights(spec, l) for l in range(len(spec.layers))]
    caches = [g.Cache.from_layer(L, w, batch) for L, w in zip(spec.layers, weights)]
    stack = g.CacheStack(caches, batch, storage="gather")
    acts = [W.activation_bulk(spec, l, labels, np.arange(batch), device="cuda") for l in range(len(spec.layers))]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        stack.run(acts)                      # eager reference (also warms everything up)
        side.synchronize()
        eager = _snapshot(stack, len(caches))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            stack.run(acts)
    assert int(eager[4][0].item()) == batch and 0 <= int(eager[4][-1].item()) <= batch
    for rep in range(4):
        # scribble over the outputs and do unrelated eager work between replays
        for t in stack.hit + stack.pred_class + stack.ids[1:]:
            t.fill_(7)
        stack.counts[1:] = -1
        junk = torch.randn(256, 256, device="cuda") @ torch.randn(256, 256, device="cuda")
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert _same(_snapshot(stack, len(caches)), eager), f"replay {rep} differs from the eager pass"
        assert torch.isfinite(junk).all()
    stack.close()
