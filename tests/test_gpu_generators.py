"""The device-side input generators produce exactly what the CPU generators do."""
import numpy as np
import pytest
import torch

from workloads import events as E
from workloads import grids as G

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("gid,name,n,first,seed", [
    (1, "g1", 432, 0, 0), (2, "g2", 100_000, 0, 0), (3, "g3", 100_001, 900_000, 0),
    (4, "g4", 77_777, 9_900_000, 0), (3, "g3", 1000, 5, 1234567)])
def test_grids(gid, name, n, first, seed):
    import paper_2404_10933_amd as M
    want = G.GRIDS[name]["make"](n=n, seed=seed, first=first)
    if name == "g1":
        want = G.grid1()
    dev = M.DeviceConfigs.empty(n)
    M.llmem_grid_generate(gid, seed, first, n, dev)
    torch.cuda.synchronize()
    got = dev.to_numpy()
    for k in want:
        assert got[k].dtype == want[k].dtype and (got[k] == want[k]).all(), k


def test_event_lists():
    import paper_2404_10933_amd as M
    n, seed, first = 3000, 7, 50_000
    ev, off = E.generate(n, seed=seed, first=first, threads=8)
    counts = torch.empty(n, dtype=torch.int64, device="cuda")
    M.llmem_events_count(seed, first, n, counts)
    offsets = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    offsets[1:] = torch.cumsum(counts, 0)
    assert (offsets.cpu().numpy() == off).all()
    events = torch.full((len(ev),), 0, dtype=torch.int64, device="cuda")
    M.llmem_events_generate(seed, first, n, offsets, events)
    torch.cuda.synchronize()
    assert (events.cpu().numpy() == ev).all()
    assert M.llmem_events_bytes(n) >= 8 * len(ev)
