"""Pins for miss compaction and stack chaining (Section 1: hits return the cached
prediction, misses continue on the base model; Appendix A.1: earlier hits remove
samples from later caches)."""
import itertools
import os

import numpy as np

from oracle import CacheDef

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_all_masks_up_to_10(oracle):
    for n in range(0, 11):
        ids = (np.arange(n, dtype=np.int32) * 7 + 3) % 101       # arbitrary distinct ids
        for mask in itertools.product((0, 1), repeat=n):
            hit = np.array(mask, np.uint8)
            got = oracle.compact_misses(hit, ids)
            assert np.array_equal(got, ids[hit == 0])             # library boolean indexing
            assert len(got) == n - int(hit.sum())


def test_properties_random(oracle):
    g = np.random.default_rng(0)
    for n in (9, 10, 63, 64, 65, 1000, 4096):
        ids = g.permutation(3 * n)[:n].astype(np.int32)
        hit = (g.random(n) < 0.4).astype(np.uint8)
        out = oracle.compact_misses(hit, ids)
        hits = ids[hit == 1]
        assert len(out) + len(hits) == n
        assert set(out.tolist()).isdisjoint(hits.tolist())
        assert set(out.tolist()) | set(hits.tolist()) == set(ids.tolist())
        pos = {v: i for i, v in enumerate(ids.tolist())}
        assert all(pos[a] < pos[b] for a, b in zip(out[:-1].tolist(), out[1:].tolist()))
        # identity ids when none are given
        assert np.array_equal(oracle.compact_misses(hit), np.nonzero(hit == 0)[0])
    assert len(oracle.compact_misses(np.ones(17, np.uint8))) == 0
    assert np.array_equal(oracle.compact_misses(np.zeros(17, np.uint8)), np.arange(17))
    assert len(oracle.compact_misses(np.zeros(0, np.uint8))) == 0
    # any non-zero byte is a hit
    assert oracle.compact_misses(np.array([0, 2, 0, 255], np.uint8)).tolist() == [0, 2]


def _read_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "effective_hit_rate.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return vals


def _threshold_cache(cut):
    """C=S=1 cache whose selector hits exactly when the single feature exceeds `cut`."""
    d = CacheDef(C=1, S=1, H=1, K=2, threshold=0.5)
    w = {"W1": np.zeros((1, 1), np.float32), "b1": np.zeros(1, np.float32),
         "W2": np.zeros((2, 1), np.float32), "b2": np.zeros(2, np.float32),
         "ws": np.array([1.0, 0.0, 0.0], np.float32), "bs": -float(cut)}
    return d, w


def test_stack_reproduces_the_papers_effective_hit_rates(oracle):
    gold = _read_golden()
    N = 1000
    g = np.random.default_rng(4)
    feat = g.permutation(N).astype(np.float32)          # distinct features 0..999, shuffled
    act = feat.reshape(N, 1, 1)
    h3 = gold["standalone_hit_block3_pool8192"] / 100.0
    h6 = gold["standalone_hit_block6_fc1024"] / 100.0
    # standalone hit sets: the top 341 features at "block 3", the top 629 at "block 6"
    d3, w3 = _threshold_cache(N - round(h3 * N) - 0.5)
    d6, w6 = _threshold_cache(N - round(h6 * N) - 0.5)
    assert oracle.lookup(d3, w3, act)["hit"].sum() == round(h3 * N)
    assert oracle.lookup(d6, w6, act)["hit"].sum() == round(h6 * N)
    res = oracle.stack([d3, d6], [w3, w6], [act, act], batch=N, storage="gather")
    new3 = int(res[0].out["hit"].sum())
    new6 = int(res[1].out["hit"].sum())
    assert abs(100.0 * new3 / N - gold["standalone_hit_block3_pool8192"]) < 1e-9
    assert abs(100.0 * new6 / N - gold["additional_hit_at_block6"]) < 1e-9
    assert abs(100.0 * len(res[1].ids_out) / N - gold["remaining_run_full_dnn"]) < 1e-9
    # the second lookup ran only on the first one's misses
    assert len(res[1].ids_in) == N - new3
    assert np.array_equal(res[1].ids_in, res[0].ids_out)
    # every request ends in exactly one place
    hit3 = res[0].ids_in[res[0].out["hit"] == 1]
    hit6 = res[1].ids_in[res[1].out["hit"] == 1]
    allv = np.concatenate([hit3, hit6, res[1].ids_out])
    assert np.array_equal(np.sort(allv), np.arange(N))


def test_stack_dense_storage_equals_gather(oracle):
    g = np.random.default_rng(8)
    N, C, S, H, K = 40, 6, 5, 7, 4
    defs, ws, acts = [], [], []
    for l in range(3):
        defs.append(CacheDef(C=C, S=S, H=H, K=K, threshold=0.5))
        ws.append({"W1": g.standard_normal((H, C)).astype(np.float32), "b1": np.zeros(H, np.float32),
                   "W2": g.standard_normal((K, H)).astype(np.float32), "b2": np.zeros(K, np.float32),
                   "ws": g.standard_normal(C + K).astype(np.float32), "bs": -0.3})
        acts.append(g.standard_normal((N, C, S)).astype(np.float32))
    ga = oracle.stack(defs, ws, acts, batch=N, storage="gather")
    dense = [acts[0]] + [np.ascontiguousarray(acts[l][ga[l - 1].ids_out]) for l in (1, 2)]
    de = oracle.stack(defs, ws, dense, batch=N, storage="dense")
    for a, b in zip(ga, de):
        assert np.array_equal(a.ids_out, b.ids_out)
        assert np.array_equal(a.out["logits"], b.out["logits"])
    assert 0 < len(ga[-1].ids_out) < N
