"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
declared symbol, and rejects bad arguments before touching the device."""
import re
import os

import numpy as np
import pytest

import paper_2101_07344_amd as g

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_is_built_and_exports_the_declared_symbols():
    lib = g.load_library()
    header = ""
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):     # every header under include/
        assert name.endswith(".h"), name
        with open(os.path.join(ROOT, "include", name)) as f:
            header += f.read()
    declared = set(re.findall(r"\b(gati_[a-z_]+)\s*\(", header))
    assert declared == set(g.exported_symbols)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings():
    seen = {g.gati_status_string(s) for s in range(5)}
    assert len(seen) == 5 and all(seen)
    assert g.gati_status_string(99)


def _weights(C, H, K):
    arrs = [np.zeros((H, C), np.float32), np.zeros(H, np.float32), np.zeros((K, H), np.float32),
            np.zeros(K, np.float32), np.zeros(C + K, np.float32)]
    return arrs, g.CacheWeights(*(a.ctypes.data for a in arrs), 0.0)


def test_create_rejects_bad_arguments_on_the_host():
    keep, w = _weights(4, 4, 4)
    good = dict(C=4, S=4, H=4, K=4, act_dtype=g.GATI_F32, layout=g.GATI_LAYOUT_NCS, threshold=0.5, max_rows=8)
    assert g.gati_cache_create(None, w)[0] == g.GATI_ERR_INVALID_ARG
    assert g.gati_cache_create(g.CacheDesc(**good), None)[0] == g.GATI_ERR_INVALID_ARG
    for key, bad in (("C", 0), ("S", -1), ("H", 0), ("K", 0), ("max_rows", 0), ("act_dtype", 7), ("layout", 3), ("selector", 5), ("predictor", 4),
                     ("threshold", float("nan"))):
        st, h = g.gati_cache_create(g.CacheDesc(**{**good, key: bad}), w)
        assert st == g.GATI_ERR_INVALID_ARG and h is None, key
    w_null = g.CacheWeights(keep[0].ctypes.data, None, keep[2].ctypes.data, keep[3].ctypes.data,
                            keep[4].ctypes.data, 0.0)
    assert g.gati_cache_create(g.CacheDesc(**good), w_null)[0] == g.GATI_ERR_INVALID_ARG
    assert g.gati_cache_create(g.CacheDesc(**{**good, "C": 1 << 21}), w)[0] == g.GATI_ERR_UNSUPPORTED
    # Pool(h): the map sizes must multiply to S, the pooled map must fit in the input map
    pool = {**good, "predictor": g.GATI_PRED_POOL_FC, "H": 0, "S": 16, "in_h": 4, "in_w": 4, "out_h": 2, "out_w": 2}
    for key, bad in (("in_h", 5), ("out_h", 0), ("out_w", 5)):
        assert g.gati_cache_create(g.CacheDesc(**{**pool, key: bad}), w)[0] == g.GATI_ERR_INVALID_ARG, key


def test_calls_reject_null_handles_and_bad_counts_on_the_host():
    assert g.gati_cache_lookup(None, 16, None, 4, None, 16, 16, 16, None, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_cache_pool(None, 16, None, 4, None, 16, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_cache_set_selector(None, 0.0, 0.5) == g.GATI_ERR_INVALID_ARG
    assert g.gati_cache_set_weights(None, g.CacheWeights()) == g.GATI_ERR_INVALID_ARG
    assert g.gati_cache_destroy(None) == g.GATI_OK
    assert g.gati_compact_misses(None, 16, None, -1, None, 16, 16, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_compact_misses(None, 16, None, 4, None, 16, None, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_compact_misses(None, None, None, 4, None, 16, 16, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_compact_misses(None, 16, 32, 4, None, 32, 16, stream=0) == g.GATI_ERR_INVALID_ARG   # in/out alias
    assert g.gati_cache_pool_variant(None) == "none"
    assert g.gati_cache_fork(None)[0] == g.GATI_ERR_INVALID_ARG
    assert g.gati_compact_misses_static(None, 16, None, -1, None, 16, 16, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_compact_misses_static(None, 16, None, g.GATI_COMPACT_STATIC_MAX_ROWS + 1, None, 16, 16, stream=0) \
        == g.GATI_ERR_UNSUPPORTED
    assert g.gati_probe_stream_read(None, 16, 16, 1, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_probe_stream_read(16, 24, 16, 1, stream=0) == g.GATI_ERR_INVALID_ARG      # not whole 16-byte vectors
    assert g.gati_probe_stream_read(16, 32, 16, 33, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_probe_copy(16, 24, 16, stream=0) == g.GATI_ERR_INVALID_ARG             # misaligned source
    assert g.gati_probe_launch_chain(None, 1, 1, 0, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_probe_launch_chain(16, 1, 0, 0, stream=0) == g.GATI_ERR_INVALID_ARG      # no workgroups
    assert g.gati_probe_launch_chain(16, 1, 1, 9, stream=0) == g.GATI_ERR_INVALID_ARG      # more dependent loads than offered
    assert g.gati_probe_launch_chain(16, 0, 1, 0, stream=0) == g.GATI_OK                   # an empty chain launches nothing


def test_trainer_calls_reject_bad_arguments_on_the_host():
    keep, w = _weights(4, 4, 4)
    good = dict(C=4, S=4, H=4, K=4, act_dtype=g.GATI_F32, layout=g.GATI_LAYOUT_NCS, threshold=0.5, max_rows=8)
    assert g.gati_trainer_create(None, w)[0] == g.GATI_ERR_INVALID_ARG
    assert g.gati_trainer_create(g.CacheDesc(**good), None)[0] == g.GATI_ERR_INVALID_ARG
    for key, bad in (("C", 0), ("H", 0), ("K", -2), ("max_rows", 0)):
        st, h = g.gati_trainer_create(g.CacheDesc(**{**good, key: bad}), w)
        assert st == g.GATI_ERR_INVALID_ARG and h is None, key
    # every predictor of the table can be trained; shapes that make no sense are refused on the host
    conv = {**good, "predictor": g.GATI_PRED_CONV_FC, "S": 16, "in_h": 4, "in_w": 4, "conv_k": 3, "conv_s": 1}
    for key, bad in (("conv_k", 5), ("conv_s", 0), ("in_h", 3), ("conv_k", 0)):
        assert g.gati_trainer_create(g.CacheDesc(**{**conv, key: bad}), w)[0] == g.GATI_ERR_INVALID_ARG, key
    assert g.gati_trainer_create(g.CacheDesc(**{**good, "predictor": 9}), w)[0] == g.GATI_ERR_INVALID_ARG
    assert g.gati_trainer_create(g.CacheDesc(**{**good, "selector": 9}), w)[0] == g.GATI_ERR_INVALID_ARG
    # the hidden-layer selector needs its three arrays and a unit count
    hid = {**good, "selector": g.GATI_SEL_HIDDEN, "selector_hidden": 8}
    assert g.gati_trainer_create(g.CacheDesc(**hid), w)[0] == g.GATI_ERR_INVALID_ARG            # Ws, cs, vs missing
    assert g.gati_trainer_get_hidden_selector(None, *(keep[:3])) == g.GATI_ERR_INVALID_ARG
    p = g.TrainParams(0.002, 0.5, 2.0)
    assert g.gati_trainer_step(None, 16, 4, 4, 16, 16, 4, p, stream=0) == g.GATI_ERR_INVALID_ARG
    assert g.gati_trainer_get_weights(None, *(keep + [np.zeros(1, np.float32)])) == g.GATI_ERR_INVALID_ARG
    assert g.gati_trainer_destroy(None) == g.GATI_OK
