"""The measurement probes shipped with the library: they must move exactly the bytes they say and leave
their buffers as documented (the bench's ceilings and counter scale factors rest on that)."""
import numpy as np
import pytest
import torch

import paper_2101_07344_amd as g

pytestmark = pytest.mark.gpu


def test_copy_probe_copies_and_read_probe_writes_nothing():
    n = (1 << 20) + 16 * 37                        # not a multiple of the grid's stride
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    assert g.gati_probe_copy(dst, src, n) == g.GATI_OK
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    sink = torch.full((256 * 32 * 1024,), -3.0, dtype=torch.float32, device="cuda")
    for shape in (0, 1, 8, 32):                    # a wave per 8 KB chunk, and three persistent grids
        assert g.gati_probe_stream_read(src, n, sink, shape) == g.GATI_OK
    torch.cuda.synchronize()
    assert bool((sink == -3.0).all())              # the sink is written only for data that cannot occur


def test_launch_chain_leaves_its_cell_zero():
    cell = torch.zeros(2, dtype=torch.int32, device="cuda")
    for wgs, loads in ((1, 0), (16, 2), (512, 8)):
        assert g.gati_probe_launch_chain(cell, 25, wgs, loads) == g.GATI_OK
    torch.cuda.synchronize()
    assert cell.cpu().tolist() == [0, 0]
