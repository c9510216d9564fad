"""Helpers shared by the GPU parity tests: run the HIP path through the binding
and bring results back as numpy arrays shaped like the oracle's."""
import numpy as np
import torch

import paper_2404_10933_amd as M


def hip_estimate(cfg_np, tables, const, detail=True, stream=None, kernel=0):
    """Returns (peaks[n], detail[n, 12] or None) computed by the HIP kernels."""
    dev = M.DeviceConfigs.from_numpy(cfg_np)
    tab = M.Tables(tables, m_base=const.m_base, cu_p=const.cu_p, align=const.align, kernel=kernel)
    n = dev.n
    peaks = torch.full((max(n, 1),), -7, dtype=torch.int64, device="cuda")
    det = torch.full((M.NDETAIL, max(n, 1)), -7, dtype=torch.int64, device="cuda") if detail else None
    M.llmem_estimate_ex(dev, tab, peaks, det, stream=stream, n=n)
    torch.cuda.synchronize()
    p = peaks.cpu().numpy()[:n]
    d = det.cpu().numpy()[:, :n].T.copy() if detail else None
    return p, d


def hip_timeline(events_np, offsets_np):
    ev = torch.from_numpy(np.ascontiguousarray(events_np, dtype=np.int64)).cuda()
    off = torch.from_numpy(np.ascontiguousarray(offsets_np, dtype=np.int64)).cuda()
    n = len(offsets_np) - 1
    a = torch.full((max(n, 1),), -7, dtype=torch.int64, device="cuda")
    r = torch.full((max(n, 1),), -7, dtype=torch.int64, device="cuda")
    M.llmem_timeline_peaks(ev, off, a, r)
    torch.cuda.synchronize()
    return a.cpu().numpy()[:n], r.cpu().numpy()[:n]


def assert_same(name, got, want):
    got, want = np.asarray(got), np.asarray(want)
    if got.shape != want.shape or not (got == want).all():
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError(f"{name}: {len(bad)} mismatches, first at {i}: got {got[i]} want {want[i]}")
