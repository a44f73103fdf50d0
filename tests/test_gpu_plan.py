"""GPU parity: fs_plan_replication (histogram + top-k under a budget) against the CPU oracle, bit-exact."""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle
from helpers import entry, random_jagged

pytestmark = pytest.mark.gpu

A, S, TAG, Z = oracle.PLAN_ACCUMULATE, oracle.PLAN_SELECT, oracle.PLAN_TAG, oracle.PLAN_ALLOW_ZERO


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def hip_plan(G, ids, offsets, T, B, row_base, R, counts_np, flags, budget=0, bpr=1, placement_np=None, n=None):
    import paper_2301_02959_amd as fs
    dev = G.DEV
    counts = torch.from_numpy(counts_np.view(np.int32).copy()).to(dev)
    ids_d = G.to_dev(ids, torch.int64) if ids is not None else None
    off_d = G.to_dev(offsets, torch.int64) if offsets is not None else None
    rb_d = G.to_dev(row_base, torch.int64) if row_base is not None else None
    if n is None:
        n = int(offsets[-1]) if offsets is not None else 0
    cap = min(R, budget // bpr) if (flags & S and bpr >= 1 and budget >= 0) else 0
    sel = torch.full((max(cap, 1),), -7, dtype=torch.int64, device=dev)
    nsel = torch.full((1,), -7, dtype=torch.int64, device=dev)
    pl = G.placement_dev(placement_np) if placement_np is not None else None
    st = torch.zeros(1, dtype=torch.int32, device=dev)
    rc = fs.fs_plan_replication(ids_d, off_d, T, B, rb_d, n, R, counts, flags, budget, bpr, sel, nsel, pl, st,
                                raise_on_error=False)
    torch.cuda.synchronize()
    k = int(nsel.item()) if flags & S and rc == 0 else 0
    return (rc, int(st.item()), counts.cpu().numpy().view(np.uint32), sel[:k].cpu().numpy(),
            pl.cpu().numpy().view(np.uint32) if pl is not None else None)


@pytest.mark.parametrize("case", [dict(T=3, B=11, E=4000, L=600), dict(T=1, B=1, E=50_000, L=200_000),
                                  dict(T=4, B=1, E=300, L=90_000)])
def test_histogram_matches(G, case):
    rng = np.random.default_rng(case["E"])
    T, B, E = case["T"], case["B"], case["E"]
    ids, offsets, row_base, n = random_jagged(rng, T, B, E, case["L"], zero_frac=0.0)
    ids = (ids.astype(np.float64) ** 3 / float(E) ** 2).astype(np.int64)       # skewed towards small ids
    base = rng.integers(0, 5, T * E).astype(np.uint32)
    oc = base.copy()
    orc, ost, _ = oracle.plan_replication(ids, offsets, T, B, row_base, T * E, oc, A)
    rc, st, hc, _, _ = hip_plan(G, ids, offsets, T, B, row_base, T * E, base, A)
    assert rc == orc == 0 and st == ost == 0
    assert np.array_equal(hc, oc) and hc.sum() - base.sum() == n


@pytest.mark.parametrize("shift,big", [(0, 1_300_001), (1, 1_300_001), (1, 40_000_001)])
def test_histogram_odd_boundaries_and_unaligned_ids(G, shift, big):
    """The histogram reads ids two at a time where it can: tables that start and end at odd positions, empty
    tables between them, an ids array that starts 8 bytes past a 16-byte boundary, a large batch whose spans
    cross tables, and ids out of range (counted as row 0 of their table, flagged) -- all as the oracle counts."""
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(11 + shift)
    T, B = 7, 1
    sizes = np.array([1, 0, 262_145, 3, 0, big, 77_777])                     # one segment per table (40 M: the large table)
    E = np.array([5, 9, 40_000, 2, 6, 900_000, 123])
    offsets = np.zeros(T + 1, np.int64)
    np.cumsum(sizes, out=offsets[1:])
    row_base = np.zeros(T + 1, np.int64)
    np.cumsum(E, out=row_base[1:])
    n, R = int(offsets[-1]), int(row_base[-1])
    ids = np.concatenate([np.minimum(rng.pareto(1.1, m).astype(np.int64), e - 1) for m, e in zip(sizes, E)])
    bad = rng.choice(n, 50, replace=False)
    ids[bad[:25]] = -1 - rng.integers(0, 1000, 25)
    ids[bad[25:]] = 10 ** 9 + rng.integers(0, 1000, 25)
    base = rng.integers(0, 3, R).astype(np.uint32)
    oc = base.copy()
    orc, ost, _ = oracle.plan_replication(ids, offsets, T, B, row_base, R, oc, A)
    assert orc == 0 and ost == oracle.BAD_ID
    buf = torch.zeros(n + 2, dtype=torch.int64, device=G.DEV)
    ids_d = buf[shift:shift + n]
    assert ids_d.data_ptr() % 16 == 8 * shift
    ids_d.copy_(torch.from_numpy(ids))
    counts = torch.from_numpy(base.view(np.int32).copy()).to(G.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    rc = fs.fs_plan_replication(ids_d, G.to_dev(offsets, torch.int64), T, B, G.to_dev(row_base, torch.int64), n, R, counts, A,
                                dev_status=st, raise_on_error=False)
    torch.cuda.synchronize()
    assert rc == 0 and int(st.item()) == oracle.BAD_ID
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), oc)


def test_histogram_zipf_profile_and_select(G):
    """c5's laws on a small table: profile, then choose under a budget, tag, and compare everything."""
    cfg = fs_inputs.CONFIGS["c5"].scaled(E=200_000, T=3)
    chunks = list(fs_inputs.make_profile_sample(cfg, per_table=400_000, device="cpu", chunk=150_000))
    R = cfg.R
    oc = np.zeros(R, np.uint32)
    hc = np.zeros(R, np.uint32)
    for t, ids_t in chunks:                      # one call per chunk: counts accumulate across calls
        ids = ids_t.numpy()
        offsets = np.zeros(cfg.T + 1, np.int64)
        offsets[t + 1:] = len(ids)
        row_base = np.arange(cfg.T + 1) * cfg.E
        orc, ost, _ = oracle.plan_replication(ids, offsets, cfg.T, 1, row_base, R, oc, A)
        rc, st, hc, _, _ = hip_plan(G, ids, offsets, cfg.T, 1, row_base, R, hc, A)
        assert rc == orc == 0 and st == ost == 0
    assert np.array_equal(hc, oc) and oc.sum() == 3 * 400_000
    pl = np.full(R, entry(2, 3), np.uint32)
    for budget_rows in (1000, int((oc > 0).sum()) + 10):       # budget binds / the non-zero rule binds
        opl, hpl = pl.copy(), pl.copy()
        orc, ost, osel = oracle.plan_replication(None, None, 1, 1, None, R, oc.copy(), S | TAG, budget_rows * 256 + 17, 256, opl)
        rc, st, _, hsel, hpl = hip_plan(G, None, None, 1, 1, None, R, oc, S | TAG, budget_rows * 256 + 17, 256, hpl)
        assert rc == orc == 0 and st == ost == 0
        assert np.array_equal(hsel, osel) and np.array_equal(hpl, opl)
        assert len(osel) == min(budget_rows, int((oc > 0).sum()))


@pytest.mark.parametrize("seed", range(3))
def test_select_ties_zeros_and_allow_zero(G, seed):
    rng = np.random.default_rng(seed)
    R = 70_001                                              # several compaction tiles + ragged tail
    counts = np.minimum(rng.pareto(1.0, R) * 2, 1e9).astype(np.uint32)      # ~1/3 zeros, heavy ties
    counts[rng.integers(0, R, 5)] = 2 ** 32 - 1
    nz = int((counts > 0).sum())
    for flags, cap in ((S, 0), (S, 1), (S, 5000), (S, nz), (S, nz + 100), (S | Z, nz + 100), (S | Z, R + 5)):
        orc, ost, osel = oracle.plan_replication(None, None, 1, 1, None, R, counts.copy(), flags, cap * 8, 8)
        rc, st, _, hsel, _ = hip_plan(G, None, None, 1, 1, None, R, counts, flags, cap * 8, 8)
        assert rc == orc == 0 and np.array_equal(hsel, osel), (flags, cap)


@pytest.mark.parametrize("shift", [0, 1, 2, 3])
def test_select_with_counts_at_any_alignment(G, shift):
    """The selection reads the counters four to a lane where their address allows it: counts arrays that start
    0, 4, 8 and 12 bytes past a 16-byte boundary give the oracle's selection, whole and in order."""
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(40 + shift)
    R = 50_003 - shift
    counts = np.minimum(rng.pareto(1.2, R) * 3, 1e6).astype(np.uint32)
    buf = torch.zeros(R + 8, dtype=torch.int32, device=G.DEV)
    view = buf[shift:shift + R]
    assert view.data_ptr() % 16 == 4 * shift
    view.copy_(torch.from_numpy(counts.view(np.int32)))
    nz = int((counts > 0).sum())
    for flags, cap in ((S, 777), (S, nz + 5), (S | Z, R)):
        orc, ost, osel = oracle.plan_replication(None, None, 1, 1, None, R, counts.copy(), flags, cap * 8, 8)
        sel = torch.full((cap,), -7, dtype=torch.int64, device=G.DEV)
        nsel = torch.full((1,), -7, dtype=torch.int64, device=G.DEV)
        st = torch.zeros(1, dtype=torch.int32, device=G.DEV)
        rc = fs.fs_plan_replication(None, None, 1, 1, None, 0, R, view, flags, cap * 8, 8, sel, nsel, None, st,
                                    raise_on_error=False)
        torch.cuda.synchronize()
        k = int(nsel.item())
        assert rc == orc == 0 and int(st.item()) == ost == 0 and k == len(osel)
        assert np.array_equal(sel[:k].cpu().numpy(), osel), (flags, cap)
    assert np.array_equal(view.cpu().numpy().view(np.uint32), counts)


def test_histogram_counts_beyond_a_table_entry_and_saturation_in_pieces(G):
    """A row met more often in one span than an entry of the kernel's LDS table can count (4096) reaches the
    global counter in pieces: the total is exact, and a counter that saturates on one of the pieces stays at
    the maximum and raises the flag, as the oracle's does."""
    rng = np.random.default_rng(77)
    R = 1000
    ids = np.concatenate([np.full(100_000, 7), np.full(10_000, 8), np.full(4096, 9), np.full(4097, 10), np.full(8192, 11),
                          rng.integers(0, R, 50_000)]).astype(np.int64)
    ids = ids[rng.permutation(len(ids))]
    offsets = np.array([0, len(ids)], np.int64)
    base = np.zeros(R, np.uint32)
    base[7] = 2 ** 32 - 5000                       # saturates part of the way
    base[8] = 2 ** 32 - 1 - 10_000 - int((ids == 8).sum() - 10_000)     # ends exactly at the maximum: no fault
    base[11] = 123
    oc = base.copy()
    orc, ost, _ = oracle.plan_replication(ids, offsets, 1, 1, [0, R], R, oc, A)
    rc, st, hc, _, _ = hip_plan(G, ids, offsets, 1, 1, [0, R], R, base, A)
    assert rc == orc == 0 and st == ost == oracle.COUNT_OVERFLOW
    assert np.array_equal(hc, oc) and hc[7] == 2 ** 32 - 1 and hc[8] == 2 ** 32 - 1 and hc[9] >= 4096 and hc[10] >= 4097


def test_saturation_faults_and_one_call_does_all(G):
    counts = np.array([2 ** 32 - 3, 0, 5, 0], np.uint32)
    orc, ost, _ = oracle.plan_replication([0, 0, 0, 0, 2], [0, 5], 1, 1, [0, 4], 4, counts.copy(), A)
    rc, st, hc, _, _ = hip_plan(G, [0, 0, 0, 0, 2], [0, 5], 1, 1, [0, 4], 4, counts, A)
    assert st == ost == oracle.COUNT_OVERFLOW and hc.tolist() == [2 ** 32 - 1, 0, 6, 0]
    rc, st, hc, _, _ = hip_plan(G, [0, 0], [0, 2], 1, 1, [0, 4], 4, counts, A)
    assert st == 0 and hc[0] == 2 ** 32 - 1
    rc, st, hc, _, _ = hip_plan(G, [9, -1, 1], [0, 3], 1, 1, [0, 4], 4, np.zeros(4, np.uint32), A)
    assert st == oracle.BAD_ID and hc.tolist() == [2, 1, 0, 0]
    rc, st, hc, _, _ = hip_plan(G, [1, 1, 1], [0, 2], 1, 1, [0, 4], 4, np.zeros(4, np.uint32), A, n=3)
    assert st == oracle.BAD_OFFSETS and hc.sum() == 0
    # accumulate + select + tag in one call
    rng = np.random.default_rng(5)
    ids, offsets, row_base, n = random_jagged(rng, 2, 30, 500, 80)
    pl = np.array([entry(2, r % 4) for r in range(1000)], np.uint32)
    oc, opl = np.zeros(1000, np.uint32), pl.copy()
    orc, ost, osel = oracle.plan_replication(ids, offsets, 2, 30, row_base, 1000, oc, A | S | TAG, 64 * 50, 64, opl)
    rc, st, hc, hsel, hpl = hip_plan(G, ids, offsets, 2, 30, row_base, 1000, np.zeros(1000, np.uint32), A | S | TAG, 64 * 50, 64, pl)
    assert rc == 0 and np.array_equal(hc, oc) and np.array_equal(hsel, osel) and np.array_equal(hpl, opl)
    # host faults
    z = np.zeros(4, np.uint32)
    assert hip_plan(G, None, None, 1, 1, None, 4, z, 16)[0] == 6
    assert hip_plan(G, None, None, 1, 1, None, 4, z, TAG)[0] == 6
    assert hip_plan(G, None, None, 1, 1, None, 4, z, S, -1, 1)[0] == 2
    assert hip_plan(G, None, None, 1, 1, None, 4, z, S, 1, 0)[0] == 2
    assert hip_plan(G, None, None, 1, 1, None, 4, z, S | TAG, 1, 1)[0] == 1
    assert hip_plan(G, None, None, 1, 1, None, 4, z, 0)[0] == 0


def test_histogram_row_base_beyond_R_drops_the_lookup(G):
    """row_base that does not fit R: the lookups it takes outside [0, R) are dropped and reported."""
    import paper_2301_02959_amd as fs
    T, B, R = 2, 3, 60
    ids = np.array([1, 2, 3, 4, 5, 6, 7, 8], dtype=np.int64)
    offsets = np.array([0, 2, 3, 4, 6, 7, 8], dtype=np.int64)     # table 0: ids[0:4], table 1: ids[4:8]
    row_base = np.array([0, 58, 70], dtype=np.int64)              # table 1 claims rows 58 .. 69, R is 60
    counts = np.zeros(R, dtype=np.uint32)
    rc, st, got, _, _ = hip_plan(G, ids, offsets, T, B, row_base, R, counts, A)
    assert rc == 0 and st & fs.FS_DEV_BAD_ID
    want = np.zeros(R, dtype=np.uint32)
    want[[1, 2, 3, 4]] = 1                                        # table 0
    assert np.array_equal(got, want)                              # 58 + 5 .. 58 + 8 are all >= 60: dropped


def test_histogram_rejects_ids_off_their_natural_alignment(G):
    """The histogram reads ids two at a time after stepping to a 16-byte boundary, which takes 8-byte aligned
    ids: an ids pointer that is not is a host fault, and nothing is launched."""
    import ctypes
    import paper_2301_02959_amd as fs
    dev = G.DEV
    ids = torch.zeros(64, dtype=torch.int64, device=dev)
    off = torch.tensor([0, 8], dtype=torch.int64, device=dev)
    rb = torch.tensor([0, 10], dtype=torch.int64, device=dev)
    counts = torch.zeros(16, dtype=torch.int32, device=dev)
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    L = fs.lib()
    P = lambda t, add=0: ctypes.c_void_p(t.data_ptr() + add)
    z = ctypes.c_void_p(0)

    def call(ids_ptr, counts_ptr):
        size = ctypes.c_size_t(ws.numel())
        return L.fs_plan_replication(ids_ptr, P(off), ctypes.c_int32(1), ctypes.c_int32(1), P(rb), ctypes.c_int64(8),
                                     ctypes.c_int64(10), counts_ptr, ctypes.c_int32(A), ctypes.c_int64(0), ctypes.c_int64(1),
                                     z, z, z, P(ws), ctypes.byref(size), z, z)
    assert call(P(ids, 4), P(counts)) == 4 and call(P(ids), P(counts, 2)) == 4
    assert call(P(ids, 8), P(counts, 4)) == 0                           # 8 mod 16 and 4 mod 16 are fine
    torch.cuda.synchronize()
    assert int(counts.sum().item()) == 8
