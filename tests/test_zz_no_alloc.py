"""gati_compact_misses_static (the entry point for callers that cannot allocate device memory)
against gati_compact_misses on the same inputs: bit-exact lists and counts, two calls in a row with
the second on a smaller input, long lists (which use the library's fixed count table) and short
ones (which need no table)."""
import numpy as np
import pytest
import torch

import paper_2101_07344_amd as g

pytestmark = pytest.mark.gpu


def _both(n, rate, seed, n_dev_val=None, with_ids=True):
    rng = np.random.default_rng(seed)
    hit = (rng.random(n) < rate).astype(np.uint8)
    ids = rng.permutation(max(2 * n, 1))[:n].astype(np.int32) if with_ids else None
    hd = torch.from_numpy(hit).cuda()
    idd = None if ids is None else torch.from_numpy(ids).cuda()
    n_dev = None if n_dev_val is None else torch.tensor([n_dev_val], dtype=torch.int32, device="cuda")
    res = []
    for fn in (g.gati_compact_misses, g.gati_compact_misses_static):
        out = torch.full((max(n, 1),), -1, dtype=torch.int32, device="cuda")
        cnt = torch.tensor([-7], dtype=torch.int32, device="cuda")
        assert fn(None, hd, idd, n, n_dev, out, cnt) == g.GATI_OK
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), int(cnt.item())))
    (a, ma), (b, mb) = res
    n_true = n if n_dev_val is None else max(0, min(n, n_dev_val))
    assert ma == mb == int((hit[:n_true] == 0).sum())
    assert np.array_equal(a, b)                       # including the untouched tail past the count
    return mb


def test_static_entry_matches_on_two_calls_in_a_row():
    # first a long list, then a shorter one: the table keeps the first call's counts, which the
    # second call must not see
    big = _both(300001, 0.3, seed=1)
    small = _both(20011, 0.9, seed=2)
    assert big > small > 0
    _both(70001, 0.0, seed=3, n_dev_val=33333)
    _both(5000, 0.5, seed=4, with_ids=False)
    _both(4096, 0.5, seed=5)                          # one-workgroup path: no table
    _both(0, 0.5, seed=6)


def test_static_entry_rejects_lists_beyond_its_table():
    d = torch.zeros(8, dtype=torch.int32, device="cuda")
    h = torch.zeros(8, dtype=torch.uint8, device="cuda")
    st = g.gati_compact_misses_static(None, h, None, g.GATI_COMPACT_STATIC_MAX_ROWS + 1, None, d, d)
    assert st == g.GATI_ERR_UNSUPPORTED
    assert "unsupported" in g.gati_status_string(st)
