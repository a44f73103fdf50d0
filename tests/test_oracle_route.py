"""Pins for the oracle's route + bucketize.

The paper fixes the tier semantics (Sections 3.1, 4.4) and that ids are
distributed to their owners before the lookup (Section 3.2, metric 2).  The
pins: brute force by a differently-written pure-Python routine on tiny inputs
over every placement; reduction to numpy's stable argsort / bincount; the
invariants; special cases with a known answer; a hand-worked example.
"""
import itertools

import numpy as np
import pytest

import oracle
from helpers import dest_numpy, entry, random_jagged, random_placement, table_of


def brute_force(ids, offsets, T, B, row_base, placement, U, W, self_):
    """Per bucket, scan all lookups in order and keep those whose destination is the bucket."""
    n = int(offsets[-1])
    lookups = []
    for i in range(n):
        seg = max(s for s in range(T * B) if offsets[s] <= i)          # last segment starting at or before i
        t = seg // B
        g = int(row_base[t] + ids[i])
        e = int(placement[g])
        tier, own = e >> 30, e & 0x3FFFFFFF
        d = self_ if tier == 0 else ((self_ // W) * W + own if tier == 1 else own)
        lookups.append((i, g, d, tier))
    rows, pos, bo = [], [], [0]
    for b in range(U):
        for (i, g, d, _) in lookups:
            if d == b:
                rows.append(g)
                pos.append(i)
        bo.append(len(rows))
    tiers = [sum(1 for l in lookups if l[3] == k) for k in range(3)]
    return bo, rows, pos, tiers


def test_hand_worked_example():
    # 2 tables of 3 rows, B = 2, U = 4, W = 2, self = 3 (group 1 = buckets 2, 3).
    # table 0: row0 tier0, row1 tier1/owner0, row2 tier2/owner1
    # table 1: row0 tier2/owner0, row1 tier1/owner1, row2 tier2/owner3
    placement = np.array([entry(0, 77), entry(1, 0), entry(2, 1), entry(2, 0), entry(1, 1), entry(2, 3)], np.uint32)
    offsets = np.array([0, 2, 3, 3, 6])           # segments: t0b0=[0,2) t0b1=[2,3) t1b0=[] t1b1=[3,6)
    ids = np.array([2, 0, 1, 2, 1, 0])
    row_base = np.array([0, 3, 6])
    # lookups: i0 g2 ->1 | i1 g0 ->3 (self) | i2 g1 ->2 | i3 g5 ->3 | i4 g4 ->3 | i5 g3 ->0
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(ids, offsets, 2, 2, row_base, placement, 4, 2, 3)
    assert rc == 0 and st == 0
    assert bo.tolist() == [0, 1, 2, 3, 6]
    assert rows.tolist() == [3, 2, 1, 0, 5, 4]
    assert pos.tolist() == [5, 0, 2, 1, 3, 4]
    assert tc.tolist() == [1, 2, 3]


@pytest.mark.parametrize("U,W", [(1, 1), (2, 1), (2, 2), (3, 1), (3, 3)])
def test_brute_force_every_placement(U, W):
    """E <= 3 rows per table, every (tier, owner) assignment, a fixed tiny batch."""
    T, B, E = 2, 2, 2
    offsets = np.array([0, 2, 2, 5, 7])
    ids = np.array([0, 1, 1, 0, 1, 0, 0])
    row_base = np.array([0, E, 2 * E])
    choices = [entry(0, 5)] + [entry(1, o) for o in range(W)] + [entry(2, o) for o in range(U)]
    for self_ in range(U):
        for combo in itertools.product(choices, repeat=T * E):
            placement = np.array(combo, np.uint32)
            rc, st, bo, rows, pos, tc = oracle.route_bucketize(ids, offsets, T, B, row_base, placement, U, W, self_)
            ebo, erows, epos, etc_ = brute_force(ids, offsets, T, B, row_base, placement, U, W, self_)
            assert rc == 0 and st == 0
            assert bo.tolist() == ebo and rows.tolist() == erows and pos.tolist() == epos
            assert tc.tolist() == etc_


@pytest.mark.parametrize("seed", range(6))
def test_reduces_to_stable_argsort(seed):
    rng = np.random.default_rng(seed)
    T, B, E = 3, 17, 50
    U, W = [(8, 4), (6, 2), (16, 16), (5, 1), (12, 3), (64, 8)][seed]
    self_ = int(rng.integers(0, U))
    ids, offsets, row_base, n = random_jagged(rng, T, B, E, 40)
    placement = random_placement(rng, T * E, U, W)
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(ids, offsets, T, B, row_base, placement, U, W, self_)
    assert rc == 0 and st == 0
    g = row_base[table_of(offsets, B)] + ids
    dest, tier = dest_numpy(g, placement, U, W, self_)
    order = np.argsort(dest, kind="stable")
    assert np.array_equal(pos, order)
    assert np.array_equal(rows, g[order])
    assert np.array_equal(bo, np.concatenate([[0], np.cumsum(np.bincount(dest, minlength=U))]))
    assert np.array_equal(tc, np.bincount(tier, minlength=3))
    # invariants (stated independently of the argsort pin)
    assert bo[-1] == n and np.array_equal(np.sort(pos), np.arange(n))
    for b in range(U):
        seg = pos[bo[b]:bo[b + 1]]
        assert np.all(np.diff(seg) > 0)
    t0 = pos[np.isin(pos, np.nonzero(tier == 0)[0])]
    lo, hi = bo[self_], bo[self_ + 1]
    assert set(t0.tolist()) <= set(pos[lo:hi].tolist())            # replicated rows served locally
    grp_lo, grp_hi = bo[(self_ // W) * W], bo[(self_ // W) * W + W]
    t1 = np.nonzero(tier == 1)[0]
    assert set(t1.tolist()) <= set(pos[grp_lo:grp_hi].tolist())    # group rows stay in the group


def test_special_cases():
    rng = np.random.default_rng(11)
    ids, offsets, row_base, n = random_jagged(rng, 2, 9, 30, 12)
    # everything replicated: one bucket, identity permutation
    placement = np.full(60, entry(0), np.uint32)
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(ids, offsets, 2, 9, row_base, placement, 4, 2, 2)
    assert bo.tolist() == [0, 0, 0, n, n] and np.array_equal(pos, np.arange(n)) and tc.tolist() == [n, 0, 0]
    # everything sharded, one bucket
    placement = np.full(60, entry(2, 0), np.uint32)
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(ids, offsets, 2, 9, row_base, placement, 1, 1, 0)
    assert bo.tolist() == [0, n] and np.array_equal(pos, np.arange(n)) and tc.tolist() == [0, 0, n]
    # contiguous-block row-wise sharding (Section 3.1): owner = id // ceil(E / U)
    U = 4
    blk = -(-30 // U)
    placement = np.array([entry(2, (r % 30) // blk) for r in range(60)], np.uint32)
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(ids, offsets, 2, 9, row_base, placement, U, 1, 1)
    for b in range(U):
        assert np.all(((rows[bo[b]:bo[b + 1]] % 30) // blk) == b)
    # empty batch
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(np.zeros(0, np.int64), np.zeros(4, np.int64), 1, 3,
                                                       np.array([0, 5]), np.zeros(5, np.uint32), 3, 1, 0)
    assert rc == 0 and st == 0 and bo.tolist() == [0, 0, 0, 0] and len(rows) == 0


def test_data_faults():
    offsets = np.array([0, 2, 4])
    row_base = np.array([0, 3, 6])
    placement = np.array([entry(2, 1), entry(2, 9), entry(3, 0), entry(1, 5), entry(0), entry(2, 0)], np.uint32)
    # id 7 is outside table 0 -> row_base[0]; id -1 outside table 1 -> row_base[1]
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(np.array([7, 1, -1, 2]), offsets, 2, 1, row_base, placement, 2, 2, 0)
    assert rc == 0 and st == (oracle.BAD_ID | oracle.BAD_PLACEMENT)
    # g = [0, 1, 3, 5]; dest: g0 ->1, g1 owner 9 >= U -> self 0, g3 tier1 owner 5 >= W -> self 0, g5 -> 0
    assert bo.tolist() == [0, 3, 4] and rows.tolist() == [1, 3, 5, 0] and pos.tolist() == [1, 2, 3, 0]
    assert tc.tolist() == [0, 1, 3]
    # tier 1: the owner must lie inside a group (< W) even when it would be a valid bucket (< U)
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(np.array([0, 1]), np.array([0, 2]), 1, 1, np.array([0, 2]),
                                                       np.array([entry(1, 5), entry(1, 1)], np.uint32), 8, 4, 6)
    assert st == oracle.BAD_PLACEMENT and bo.tolist() == [0, 0, 0, 0, 0, 0, 1, 2, 2] and rows.tolist() == [1, 0]
    # tier 3 counts under tier 0 and is served locally
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(np.array([2]), np.array([0, 1]), 1, 1, np.array([0, 3]), placement[:3], 2, 1, 1)
    assert st == oracle.BAD_PLACEMENT and bo.tolist() == [0, 0, 1] and tc.tolist() == [1, 0, 0]
    # offsets: decreasing, wrong start, wrong end
    for bad in ([0, 3, 2], [1, 2, 4], [0, 2, 5]):
        rc, st, *_ = oracle.route_bucketize(np.array([0, 1, 2, 0]), np.array(bad), 2, 1, row_base, placement, 2, 2, 0, n=4)
        assert rc == 0 and st & oracle.BAD_OFFSETS


def test_host_faults():
    ids, offsets, row_base = np.array([0]), np.array([0, 1]), np.array([0, 2])
    pl = np.zeros(2, np.uint32)
    call = lambda **kw: oracle.route_bucketize(ids, offsets, kw.get("T", 1), kw.get("B", 1), row_base, pl,
                                               kw.get("U", 2), kw.get("W", 1), kw.get("s", 0), n=kw.get("n", 1))[0]
    assert call() == 0
    assert call(n=-1) == 2 and call(T=0) == 2 and call(B=0) == 2
    assert call(U=0) == 6 and call(U=4097) == 6 and call(W=0) == 6 and call(U=4, W=3) == 6
    assert call(s=2) == 6 and call(s=-1) == 6
