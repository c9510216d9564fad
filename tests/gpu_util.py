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


def _tp_tensor(tp_np):
    return None if tp_np is None else torch.from_numpy(np.ascontiguousarray(tp_np, dtype=np.uint8)).cuda()


def hip_methods(cfg_np, tp_np, tables, const, flags=True, stream=None):
    """Returns (peaks[n, 4], flags[n] or None): the four methods' estimates by the HIP kernel."""
    dev = M.DeviceConfigs.from_numpy(cfg_np)
    tab = M.Tables(tables, m_base=const.m_base, cu_p=const.cu_p, align=const.align)
    n = dev.n
    peaks = torch.full((4, max(n, 1)), -7, dtype=torch.int64, device="cuda")
    fl = torch.full((max(n, 1),), -7, dtype=torch.int64, device="cuda") if flags else None
    M.llmem_estimate_methods(dev, _tp_tensor(tp_np), tab, peaks, fl, stream=stream, n=n)
    torch.cuda.synchronize()
    return peaks.cpu().numpy()[:, :n].T.copy(), (fl.cpu().numpy()[:n] if flags else None)


def hip_decide(cfg_np, tp_np, tables, const, m_total, detail=True, short=True, stream=None):
    """Returns (method[n], bs[n], rows[n, 12] or None): Algorithm 1 by the HIP kernel."""
    dev = M.DeviceConfigs.from_numpy(cfg_np)
    tab = M.Tables(tables, m_base=const.m_base, cu_p=const.cu_p, align=const.align)
    n = dev.n
    method = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda") if short else None
    bs = torch.full((max(n, 1),), -7, dtype=torch.int32, device="cuda") if short else None
    det = torch.full((M.NDECIDE, max(n, 1)), -7, dtype=torch.int64, device="cuda") if detail else None
    M.llmem_decide(dev, _tp_tensor(tp_np), tab, m_total, method, bs, det, stream=stream, n=n)
    torch.cuda.synchronize()
    return (method.cpu().numpy()[:n] if short else None, bs.cpu().numpy()[:n] if short else None,
            det.cpu().numpy()[:, :n].T.copy() if detail else None)


def hip_sweep(grid_id, seed, first, n, tables, const, m_total, kernel=0, into=None, stream=None):
    """Returns stats[NSWEEP, SWEEP_GROUPS] of a sweep by the HIP kernel; `into`: a device
    array to go on accumulating into (else a freshly reset one)."""
    tab = M.Tables(tables, m_base=const.m_base, cu_p=const.cu_p, align=const.align, kernel=kernel)
    stats = into
    if stats is None:
        stats = torch.full((M.NSWEEP, M.SWEEP_GROUPS), -7, dtype=torch.int64, device="cuda")
        M.llmem_sweep_reset(stats, stream=stream)
    M.llmem_sweep(grid_id, seed, first, n, tab, m_total, stats, stream=stream)
    torch.cuda.synchronize()
    return stats if into is not None else stats.cpu().numpy()
