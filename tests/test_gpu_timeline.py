"""Parity of the explicit-timeline kernel with the CPU oracle (bit exact)."""
import numpy as np
import pytest
import torch

from oracle import llmem_oracle as A
from oracle import oracle_c as B
from workloads import events as E

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def U():
    import gpu_util
    return gpu_util


def _check(U, ev, off):
    want_a, want_r = B.event_lists_peaks(ev, off, threads=8)
    got_a, got_r = U.hip_timeline(ev, off)
    U.assert_same("allocated", got_a, want_a)
    U.assert_same("reserved", got_r, want_r)


def test_handwritten_lists(U):
    M2 = 2 * 1024 * 1024
    lists = [[], [1], [-1, 1], [511, 512, 513, -511, -512, -513], [M2 - 513, M2 - 512, M2 - 511, M2, M2 + 1],
             [3_000_000, 100, -3_000_000, 100], [0, 0, 0], [5, -5] * 700, [M2] * 1500 + [-M2] * 1500,
             list(range(1, 1024)), list(range(1, 1025)), list(range(1, 1026)), list(range(1, 2050)), [],
             [-600], [-600, 100], [-3_000_000, 100]]              # nothing live before the first event: peaks of zero
    ev, off = E.from_lists(lists)
    _check(U, ev, off)
    a, r = A.event_lists_peaks(ev, off)                  # the pinned Python oracle agrees too
    got_a, got_r = U.hip_timeline(ev, off)
    assert list(got_a) == a and list(got_r) == r


def test_random_ragged_lists(U):
    rng = np.random.default_rng(21)
    lists = []
    for _ in range(300):
        n = int(rng.integers(0, 5000))
        mag = (2.0 ** rng.uniform(0, 24, size=n)).astype(np.int64)
        lists.append(list(np.where(rng.random(n) < 0.5, mag, -mag)))   # arbitrary signs: prefixes go negative
    ev, off = E.from_lists(lists)
    _check(U, ev, off)
    # the event array at every 8-byte position within a 128-byte line (the kernel reads whole lines)
    import paper_2404_10933_amd as M
    want_a, want_r = B.event_lists_peaks(ev, off, threads=8)
    n = len(off) - 1
    off_dev = torch.from_numpy(off).cuda()
    for shift in (1, 2, 7, 15):
        padded = torch.full((len(ev) + 32,), 1 << 40, dtype=torch.int64, device="cuda")    # what surrounds the lists must not count
        padded[shift:shift + len(ev)] = torch.from_numpy(ev).cuda()
        a = torch.full((n,), -7, dtype=torch.int64, device="cuda")
        r = torch.full((n,), -7, dtype=torch.int64, device="cuda")
        M.llmem_timeline_peaks(padded[shift:shift + len(ev)], off_dev, a, r)
        torch.cuda.synchronize()
        U.assert_same(f"allocated, array shifted by {shift}", a.cpu().numpy(), want_a)
        U.assert_same(f"reserved, array shifted by {shift}", r.cpu().numpy(), want_r)


def test_wide_events_take_the_64_bit_path(U):
    """Events of 2^35 bytes and more leave the 32-bit block-count walk; mix both
    kinds inside and across tiles, at both sides of the threshold."""
    rng = np.random.default_rng(22)
    T35 = 1 << 35
    lists = [[T35 - 1, -(T35 - 1)], [T35, -T35], [T35 + 1, 5, -(T35 + 1)], [-T35, -(T35 - 1), T35 - 511, T35 - 512]]
    for _ in range(120):
        n = int(rng.integers(1, 4000))
        mag = (2.0 ** rng.uniform(0, 30, size=n)).astype(np.int64)
        wide = rng.random(n) < rng.choice((0.0, 0.001, 0.05, 1.0))
        mag = np.where(wide, (2.0 ** rng.uniform(35, 50, size=n)).astype(np.int64), mag)
        lists.append(list(np.where(rng.random(n) < 0.5, mag, -mag)))
    ev, off = E.from_lists(lists)
    _check(U, ev, off)


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 257])
def test_generated_lists_small(U, n):
    ev, off = E.generate(n, seed=2, first=11, threads=8)
    _check(U, ev, off)


def test_full_size_event_grid(U):
    """10^5 lists of about 10^4 events (8 GB), every list against the oracle."""
    n = 100_000
    ev, off = E.generate(n, seed=0, threads=16)
    assert len(ev) > 9 * 10 ** 8
    _check(U, ev, off)
