"""Whole-batch parity at the BASELINE batch sizes, in the launch configuration bench.py times
(device-chained fused stack over GPU-drawn tensors): EVERY row the library looks up at EVERY
layer is compared with the CPU oracle.

Per layer the oracle looks up exactly the rows the library looked up (its incoming miss list):
  * logits and confidence of every row, within the fp32 / bf16 bounds (bf16: against the oracle
    with the same operand rounding, and against the unrounded arithmetic);
  * class and hit flag bit-exact on every row whose oracle margins (top-2 logit gap, distance of
    the confidence from the threshold) are at least 1e-3 -- the bulk tensors are not redrawn for
    admissibility, so the test also requires that at least 95 % of the rows are that sure;
  * the outgoing miss list bit-exact against the oracle's own chain for as long as no unsure row
    was decided differently, and always equal to the oracle's stable compaction of the library's
    own hit flags with the count in device memory.
The oracle stays single-threaded per call; the harness runs independent row shards of a layer on
several host threads (ctypes releases the interpreter lock), which changes no value.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import paper_2101_07344_amd as g
import workloads as W
from oracle import admit

from helpers import TOL, TOL_MIRROR_BF16, ideal_def

pytestmark = pytest.mark.gpu

MARGIN = 1e-3
# bf16 caches against the oracle with the same operand rounding.  The two sides round the pooled mean
# and the hidden vector to bf16 from values that differ in the last fp32 bits (fp32 tree sum against an
# fp64 sum), so now and then an operand sits on a rounding boundary and lands one bf16 step apart: a
# step of the hidden value h_j moves logit k by ulp_bf16(h_j) |W2[k,j]|, about 2e-3 at these shapes,
# and a step of a pooled mean moves every hidden unit of its row a little, which flips a few of them.
# Among the 10^6..10^7 logits of a full batch a handful of rows collect several such steps, so the
# whole-batch bound is 1e-2 on the largest error with at most 0.1 % of the rows beyond the 5e-3 that
# the small parity cases hold; the bound against the unrounded arithmetic stays the stated 2e-2.
TOL_MIRROR_WHOLE_BATCH = 1e-2
ROWS_BEYOND_SMALL_CASE_BOUND = 1e-3
HOST_THREADS = max(1, min(16, os.cpu_count() or 1))


def oracle_rows(d, w, act_host, rows):
    """oracle.lookup of the given rows of act_host, sharded over host threads; rows in order."""
    rows = np.ascontiguousarray(rows, np.int32)
    if len(rows) == 0:
        return oracle.lookup(d, w, act_host, row_index=rows, n=0)
    shards = [s for s in np.array_split(rows, min(HOST_THREADS, len(rows))) if len(s)]
    with ThreadPoolExecutor(len(shards)) as ex:
        outs = list(ex.map(lambda s: oracle.lookup(d, w, act_host, row_index=s, n=len(s)), shards))
    return {k: np.concatenate([o[k] for o in outs]) for k in outs[0]}


class Tally:
    def __init__(self):
        self.rows = self.sure = self.rows_beyond = 0
        self.max_err = {"logits": 0.0, "confidence": 0.0, "logits_ideal": 0.0, "confidence_ideal": 0.0}
        self.diverged_at = None


def compare_layer(l, L, d, w, act_host, rows_in_act, ids_in, got, ids_next, n_next, oracle_ids, tally):
    """One layer, all n active rows.  rows_in_act[i]: row of act_host that active row i reads.
    oracle_ids: the oracle's own incoming miss list, or None once the two chains may differ.
    Returns the oracle's outgoing list (or None)."""
    n = len(ids_in)
    want = oracle_rows(d, w, act_host, rows_in_act)
    bf16 = L.dtype == "bf16"
    tol = TOL_MIRROR_WHOLE_BATCH if bf16 else TOL["f32"]
    if n:
        row_err = np.max(np.abs(got["logits"][:n].astype(np.float64) - want["logits"]), axis=1)
        ez = float(row_err.max())
        ec = float(np.max(np.abs(got["confidence"][:n].astype(np.float64) - want["confidence"])))
        if bf16:
            tally.rows_beyond += int((row_err > TOL_MIRROR_BF16).sum())
        tally.max_err["logits"] = max(tally.max_err["logits"], ez)
        tally.max_err["confidence"] = max(tally.max_err["confidence"], ec)
        assert ez <= tol, f"layer {l}: logits max abs err {ez} > {tol}"
        assert ec <= tol, f"layer {l}: confidence max abs err {ec} > {tol}"
        if bf16:
            ideal = oracle_rows(ideal_def(d), w, act_host, rows_in_act)
            ez = float(np.max(np.abs(got["logits"][:n].astype(np.float64) - ideal["logits"])))
            ec = float(np.max(np.abs(got["confidence"][:n].astype(np.float64) - ideal["confidence"])))
            tally.max_err["logits_ideal"] = max(tally.max_err["logits_ideal"], ez)
            tally.max_err["confidence_ideal"] = max(tally.max_err["confidence_ideal"], ec)
            assert ez <= TOL["bf16"], f"layer {l}: logits vs unrounded arithmetic {ez} > {TOL['bf16']}"
            assert ec <= TOL["bf16"], f"layer {l}: confidence vs unrounded arithmetic {ec} > {TOL['bf16']}"
    z = np.sort(want["logits"].astype(np.float64), axis=1)
    gap = z[:, -1] - z[:, -2] if z.shape[1] > 1 else np.full(n, np.inf)
    dist = np.abs(want["confidence"].astype(np.float64) - d.threshold)
    sure_c, sure_h = gap >= MARGIN, dist >= MARGIN
    tally.rows += n
    tally.sure += int((sure_c & sure_h).sum())
    assert np.array_equal(got["pred_class"][:n][sure_c], want["pred_class"][sure_c]), f"layer {l}: class"
    assert np.array_equal(got["hit"][:n][sure_h], want["hit"][sure_h]), f"layer {l}: hit"
    # the outgoing list: always the stable compaction of the library's own flags ...
    assert n_next == int((got["hit"][:n] == 0).sum()), f"layer {l}: miss count"
    assert np.array_equal(ids_next[:n_next], oracle.compact_misses(got["hit"][:n], ids_in)), f"layer {l}: miss list"
    # ... and bit-exact against the oracle's own chain until an unsure row is decided differently
    if oracle_ids is not None:
        assert np.array_equal(ids_in, oracle_ids), f"layer {l}: incoming list differs from the oracle's chain"
        if np.array_equal(got["hit"][:n], want["hit"]):
            out = oracle.compact_misses(want["hit"], ids_in)
            assert np.array_equal(ids_next[:n_next], out), f"layer {l}: miss list vs the oracle's chain"
            return out
        tally.diverged_at = l
    return None


def outputs_of(stack, l):
    return {"logits": stack.logits[l].cpu().numpy(), "confidence": stack.confidence[l].cpu().numpy(),
            "pred_class": stack.pred_class[l].cpu().numpy(), "hit": stack.hit[l].cpu().numpy()}


@pytest.mark.parametrize("name", ["resnet18", "resnet50", "bert_base"])
def test_every_row_of_every_layer(name):
    spec = W.get_workload(name)
    n_layers = len(spec.layers)
    labels = W.zipf_labels(spec.batch, spec.layers[0].K, spec.zipf_s, spec.seed)
    weights = [W.cache_weights(spec, l) for l in range(n_layers)]
    caches = [g.Cache.from_layer(L, w, spec.batch) for L, w in zip(spec.layers, weights)]
    defs = admit.cache_defs(spec, mirror=True)
    acts = [W.activation_bulk(spec, l, labels, np.arange(spec.batch), device="cuda") for l in range(n_layers)]
    # the timed configuration keeps no logits; its decisions must equal those of the pass that does
    plain = g.CacheStack(caches, spec.batch, storage="gather", keep_logits=False)
    plain.run(acts)
    torch.cuda.synchronize()
    stack = g.CacheStack(caches, spec.batch, storage="gather", keep_logits=True)
    stack.run(acts)
    torch.cuda.synchronize()
    counts = stack.counts.cpu().numpy()
    assert np.array_equal(counts, plain.counts.cpu().numpy())
    tally, oracle_ids = Tally(), np.arange(spec.batch, dtype=np.int32)
    assert counts[0] == spec.batch
    for l in range(n_layers):
        n, m = int(counts[l]), int(counts[l + 1])
        for a, b in ((stack.pred_class, plain.pred_class), (stack.confidence, plain.confidence), (stack.hit, plain.hit),
                     (stack.ids, plain.ids)):
            assert torch.equal(a[l][:n], b[l][:n]), f"layer {l}: pass without logits differs"
        ids_in = stack.ids[l].cpu().numpy()[:n]
        act_host = W.to_host_array(acts[l])
        oracle_ids = compare_layer(l, spec.layers[l], defs[l], weights[l], act_host, ids_in, ids_in, outputs_of(stack, l),
                                   stack.ids[l + 1].cpu().numpy(), m, oracle_ids, tally)
        del act_host
    print(f"\n[{name}] {tally.rows} lookups compared, {tally.sure} sure ({tally.sure / tally.rows:.4f}), "
          f"max errors {tally.max_err}, rows beyond {TOL_MIRROR_BF16}: {tally.rows_beyond}, chains identical through layer "
          f"{n_layers - 1 if tally.diverged_at is None else tally.diverged_at - 1}")
    assert tally.rows == int(counts[:n_layers].sum())
    assert tally.sure >= 0.95 * tally.rows
    assert tally.rows_beyond <= ROWS_BEYOND_SMALL_CASE_BOUND * tally.rows, tally.rows_beyond
    hit_total = spec.batch - int(counts[n_layers])
    assert 0.3 * spec.batch < hit_total < 0.95 * spec.batch
    stack.close()


def test_resnet152_first_layers_every_row():
    """Layers 0-3 of the streaming 4096-request stack (dense storage: each layer holds only the
    rows still active, in miss-list order), one layer at a time so that one 6.6 GB tensor lives
    on the host at once."""
    base = W.get_workload("resnet152")
    spec = W.WorkloadSpec(name="resnet152[0:4]", batch=base.batch, zipf_s=base.zipf_s, seed=base.seed,
                          layers=base.layers[:4], storage="dense")
    labels = W.zipf_labels(spec.batch, spec.layers[0].K, spec.zipf_s, spec.seed)
    weights = [W.cache_weights(spec, l) for l in range(4)]
    caches = [g.Cache.from_layer(L, w, spec.batch) for L, w in zip(spec.layers, weights)]
    defs = admit.cache_defs(spec, mirror=True)
    stack = g.CacheStack(caches, spec.batch, storage="dense", keep_logits=True)
    tally, oracle_ids = Tally(), np.arange(spec.batch, dtype=np.int32)
    active = np.arange(spec.batch)
    for l in range(4):
        act = W.activation_bulk(spec, l, labels, active, device="cuda")
        stack.run_layer(l, act)
        torch.cuda.synchronize()
        counts = stack.counts.cpu().numpy()
        n, m = int(counts[l]), int(counts[l + 1])
        assert n == len(active)
        ids_in = stack.ids[l].cpu().numpy()[:n]
        act_host = W.to_host_array(act)
        del act
        oracle_ids = compare_layer(l, spec.layers[l], defs[l], weights[l], act_host, np.arange(n, dtype=np.int32), ids_in,
                                   outputs_of(stack, l), stack.ids[l + 1].cpu().numpy(), m, oracle_ids, tally)
        del act_host
        active = stack.ids[l + 1][:m].cpu().numpy().astype(np.int64)
    print(f"\n[resnet152 layers 0-3] {tally.rows} lookups compared, {tally.sure} sure, max errors {tally.max_err}, "
          f"rows beyond {TOL_MIRROR_BF16}: {tally.rows_beyond}")
    assert tally.sure >= 0.95 * tally.rows
    assert tally.rows_beyond <= ROWS_BEYOND_SMALL_CASE_BOUND * tally.rows, tally.rows_beyond
    stack.close()
