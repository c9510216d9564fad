"""The seeded inputs: structure of the default tables, the counter hash shared
by the numpy and C generators, grid field ranges, event-list well-formedness."""
import numpy as np

from workloads import events as E
from workloads import grids as G
from workloads import tables as T


def test_default_tables_are_balanced():
    """One iteration of each family returns to zero live activations and never
    goes negative, for every method (sizes unrounded; pure bookkeeping check)."""
    D = dict(one=1, bs=3, sl=17, sl_m1=16, h=64, ffn=172, n_heads=4, n_kv=2, head_dim=16, kv_dim=32,
             V=1000, P=40, L=5, B_logits=4, d=3)
    for fam, make, checkpoint in [(f, m, c) for f, m in T.FAMILIES.items() for c in (True, False)]:
        t = make(checkpoint=checkpoint)
        assert (250 if checkpoint else 190) <= len(t.events) <= 400
        segs = [e.seg for e in t.events]
        assert segs == sorted(segs, key=T.SEGMENTS.index)
        for method in (0, 1, 2):
            live = 0
            for s in ["A"] + ["F"] * D["L"] + ["H"] + ["B"] * D["L"] + ["Z"]:
                for e in t.events:
                    if e.seg != s or method not in e.methods:
                        continue
                    v = e.coef * e.elem_bytes
                    for name in e.dims:
                        v *= D[name]
                    if e.scale == "tp_gather":
                        v = -(-v * (D["d"] - 1) // D["d"])
                    live += e.sign * v * (D["L"] if e.times_L else 1)
                    assert live >= 0
            assert live == 0


def test_uncheckpointed_tables_keep_what_autograd_saves():
    """Without checkpointing the forward of a block frees nothing that autograd saved: its net
    change is the block output plus the saved tensors, far above the checkpointed block's one
    kept output; the parameter entries are the same."""
    for fam, make in T.FAMILIES.items():
        full, ckpt = make(checkpoint=False), make()
        assert full.params == ckpt.params and full.name == ckpt.name + "_full"
        net = lambda t: sum(e.sign for e in t.events if e.seg == "F")
        assert net(ckpt) == 1 and net(full) >= 15
        # no recomputation: the backward segment holds no forward operator
        assert not any(e.name.startswith("re:") for e in full.events)
        assert any(e.name.startswith("re:") for e in ckpt.events)


def test_grid_shapes_and_ranges():
    g1 = G.grid1()
    assert len(g1["bs"]) == 432 and len({tuple(int(g1[k][i]) for k in g1) for i in range(432)}) == 432
    g2 = G.grid2(n=5000)
    assert set(np.unique(g2["h"])) <= {768, 1024, 2048, 2560, 4096}
    assert g2["L"].min() >= 12 and g2["L"].max() <= 32 and (g2["ffn"] == 4 * g2["h"]).all()
    assert set(np.unique(g2["d"])) == set(range(1, 17)) and set(np.unique(g2["method"])) == {0, 1, 2}
    g4 = G.grid4(n=5000)
    assert (g4["chunk_k"] == -1).all() and set(np.unique(g4["n_kv"])) == {1, 4, 8}
    assert set(np.unique(g4["sl"])) == {512, 1024, 2048, 4096, 8192}
    for name, dt in G.FIELDS:
        assert g4[name].dtype == dt
    # slices of a grid are reproducible independently
    a, b = G.grid3(n=100, first=50), G.grid3(n=1000)
    assert all((a[k] == b[k][50:150]).all() for k in a)


def test_hash_agrees_between_numpy_and_c():
    idx = np.arange(64, dtype=np.uint64)
    n_fwd = 2800 + G.mix64(5, idx + np.uint64(9), 100) % np.uint64(651)
    n_saved = np.zeros(64, dtype=np.int64)
    for i in range(64):
        j = np.arange(int(n_fwd[i]), dtype=np.uint64) + np.uint64((9 + i) * 8192)
        n_saved[i] = int(((G.mix64(5, j, 103) % np.uint64(10)) < 3).sum())
    assert (E.counts(64, seed=5, first=9) == 2 * n_fwd.astype(np.int64) + 4 * n_saved).all()
    assert int(G.mix64(0, np.zeros(1, dtype=np.uint64), 0)[0]) == _mix_scalar(0, 0, 0)


def _mix_scalar(seed, index, field):
    m = (1 << 64) - 1
    x = (seed + 0x9E3779B97F4A7C15 * (index + 1) + 0xD1B54A32D192ED03 * (field + 1)) & m
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & m
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & m
    x ^= x >> 31
    return x


def test_event_lists_are_well_formed():
    ev, off = E.generate(50, seed=1, first=3, threads=2)
    assert off[0] == 0 and off[-1] == len(ev)
    lens = np.diff(off)
    assert lens.min() >= 2 * 2800 and lens.max() <= 2 * 3450 + 4 * 3450 and 9000 < lens.mean() < 11000
    for i in range(50):
        s = np.cumsum(ev[off[i]:off[i + 1]])
        assert s.min() >= 0 and s[-1] == 0
    mag = np.abs(ev)
    assert mag.min() >= 32 and mag.max() < 2 ** 28 and (mag % 512 != 0).mean() > 0.9
    ev2, off2 = E.generate(10, seed=1, first=13)
    assert (ev2 == ev[off[10]:off[20]]).all()


def test_query_grid():
    cfg, tp = G.grid6(n=5000, seed=3, first=10)
    d = cfg["d"].astype(int)
    assert set(np.unique(d)) == {1, 2, 4, 8, 16}
    assert (tp >= 1).all() and (d % tp == 0).all() and ((tp & (tp - 1)) == 0).all()
    assert (cfg["bs"] == G.QUERY_BS_CAP).all() and (cfg["chunk_k"] == G.CHUNK_SEARCH).all()
    # same model shapes as grid 4, slice-independent
    g4 = G.grid4(n=5000, seed=3, first=10)
    for k in ("h", "L", "n_heads", "n_kv", "ffn", "V", "sl", "flags"):
        assert (cfg[k] == g4[k]).all()
    part, tp_part = G.grid6(n=100, seed=3, first=110)
    assert (part["d"] == cfg["d"][100:200]).all() and (tp_part == tp[100:200]).all()
    # every admissible (gpu_n, tp_n) pair occurs
    assert len({(int(a), int(b)) for a, b in zip(d, tp)}) == 15
