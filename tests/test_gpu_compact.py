"""GPU parity of miss compaction (integer work: bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2101_07344_amd as g

pytestmark = pytest.mark.gpu


def _run(hit, ids, n_max=None, n_dev_val=None):
    n = len(hit)
    n_max = n if n_max is None else n_max
    hd = torch.from_numpy(hit).cuda()
    idd = None if ids is None else torch.from_numpy(ids).cuda()
    out = torch.full((max(n_max, 1),), -1, dtype=torch.int32, device="cuda")
    cnt = torch.tensor([-5], dtype=torch.int32, device="cuda")
    n_dev = None if n_dev_val is None else torch.tensor([n_dev_val], dtype=torch.int32, device="cuda")
    st = g.gati_compact_misses(None, hd, idd, n_max, n_dev, out, cnt)
    assert st == g.GATI_OK
    torch.cuda.synchronize()
    return out.cpu().numpy(), int(cnt.item())


@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 65, 256, 1023, 1024, 1025, 2047, 4096, 4097, 5000, 8193, 70001, 1048577, 4200000])
@pytest.mark.parametrize("rate", [0.0, 0.3, 1.0])
def test_compaction_matches_oracle(n, rate):
    rng = np.random.default_rng(n * 3 + int(rate * 10))
    hit = (rng.random(n) < rate).astype(np.uint8)
    hit[hit == 1] = rng.integers(1, 256, size=int(hit.sum())).astype(np.uint8)   # any non-zero byte
    ids = rng.permutation(max(2 * n, 1))[:n].astype(np.int32)
    want = oracle.compact_misses(hit, ids)
    out, m = _run(hit, ids)
    assert m == len(want)
    assert np.array_equal(out[:m], want)
    assert np.all(out[m:] == -1)                      # nothing written past the count
    want_id = oracle.compact_misses(hit, None)
    out, m = _run(hit, None)
    assert m == len(want_id) and np.array_equal(out[:m], want_id)


def test_device_count_and_aliasing():
    rng = np.random.default_rng(1)
    hit = (rng.random(3000) < 0.5).astype(np.uint8)
    ids = np.arange(3000, dtype=np.int32)[::-1].copy()
    out, m = _run(hit, ids, n_max=3000, n_dev_val=1500)
    want = oracle.compact_misses(hit[:1500], ids[:1500])
    assert m == len(want) and np.array_equal(out[:m], want)
    # count in and count out in the same device scalar
    hd, idd = torch.from_numpy(hit).cuda(), torch.from_numpy(ids).cuda()
    outd = torch.zeros(3000, dtype=torch.int32, device="cuda")
    cnt = torch.tensor([2000], dtype=torch.int32, device="cuda")
    assert g.gati_compact_misses(None, hd, idd, 3000, cnt, outd, cnt) == g.GATI_OK
    torch.cuda.synchronize()
    want = oracle.compact_misses(hit[:2000], ids[:2000])
    assert int(cnt.item()) == len(want)
    assert np.array_equal(outd.cpu().numpy()[:len(want)], want)


def test_long_list_device_count_and_aliasing():
    """Lists beyond one workgroup's reach (two launches over many workgroups): a device-side count
    that ends inside a span, and the count read and written through one device scalar."""
    rng = np.random.default_rng(7)
    n_max = 50000
    hit = (rng.random(n_max) < 0.4).astype(np.uint8)
    ids = rng.permutation(n_max).astype(np.int32)
    for n_true in (0, 1, 4096, 4097, 33333, 50000, 60000):
        out, m = _run(hit, ids, n_max=n_max, n_dev_val=n_true)
        want = oracle.compact_misses(hit[:min(n_true, n_max)], ids[:min(n_true, n_max)])
        assert m == len(want) and np.array_equal(out[:m], want), n_true
        assert np.all(out[m:] == -1)
    hd, idd = torch.from_numpy(hit).cuda(), torch.from_numpy(ids).cuda()
    outd = torch.zeros(n_max, dtype=torch.int32, device="cuda")
    cnt = torch.tensor([41234], dtype=torch.int32, device="cuda")
    assert g.gati_compact_misses(None, hd, idd, n_max, cnt, outd, cnt) == g.GATI_OK
    torch.cuda.synchronize()
    want = oracle.compact_misses(hit[:41234], ids[:41234])
    assert int(cnt.item()) == len(want)
    assert np.array_equal(outd.cpu().numpy()[:len(want)], want)
