"""Pins for the oracle's replication plan (Section 4.1: per-row appearance
counts; Section 4.3: descending-frequency prefix under a memory budget;
Section 4.6: tables merged into one distribution) and for the few numbers the
paper prints that touch this path (tests/golden/paper_tables.txt).
"""
import os

import numpy as np
import pytest

import oracle
from helpers import entry, random_jagged, table_of

A, S, TAG, Z = oracle.PLAN_ACCUMULATE, oracle.PLAN_SELECT, oracle.PLAN_TAG, oracle.PLAN_ALLOW_ZERO


def golden():
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_tables.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = [s.strip() for s in line.split("=")]
                out[k] = float(v) if "." in v else int(v)
    return out


@pytest.mark.parametrize("seed", range(3))
def test_histogram_is_bincount(seed):
    rng = np.random.default_rng(seed)
    T, B, E = 3, 11, 40
    ids, offsets, row_base, n = random_jagged(rng, T, B, E, 30)
    g = row_base[table_of(offsets, B)] + ids
    counts = np.zeros(T * E, np.uint32)
    rc, st, _ = oracle.plan_replication(ids, offsets, T, B, row_base, T * E, counts, A)
    assert rc == 0 and st == 0
    assert np.array_equal(counts, np.bincount(g, minlength=T * E))
    assert counts.sum() == n                                   # sum of frequencies = number of lookups (eq. 2, unnormalised)
    rc, st, _ = oracle.plan_replication(ids, offsets, T, B, row_base, T * E, counts, A)
    assert np.array_equal(counts, 2 * np.bincount(g, minlength=T * E))   # calls accumulate


def test_histogram_saturates():
    counts = np.array([2 ** 32 - 3, 0, 5], np.uint32)
    rc, st, _ = oracle.plan_replication([0, 0, 0, 0, 2], [0, 5], 1, 1, [0, 3], 3, counts, A)
    assert st == oracle.COUNT_OVERFLOW and counts.tolist() == [2 ** 32 - 1, 0, 6]
    counts = np.array([2 ** 32 - 3, 0, 5], np.uint32)
    rc, st, _ = oracle.plan_replication([0, 0], [0, 2], 1, 1, [0, 3], 3, counts, A)
    assert st == 0 and counts[0] == 2 ** 32 - 1                # reaching the maximum exactly is not an overflow
    counts = np.zeros(3, np.uint32)
    rc, st, _ = oracle.plan_replication([5, -1], [0, 2], 1, 1, [0, 3], 3, counts, A)
    assert st == oracle.BAD_ID and counts.tolist() == [2, 0, 0]                                  # out-of-table ids count on the table's first row


@pytest.mark.parametrize("seed", range(4))
def test_select_is_lexsort_prefix(seed):
    rng = np.random.default_rng(100 + seed)
    R = 500
    counts = np.minimum(rng.pareto(1.0, R) * 3, 1e6).astype(np.uint32)   # many ties, many zeros
    order = np.lexsort((np.arange(R), -counts.astype(np.int64)))
    nz = int((counts > 0).sum())
    for cap in (0, 1, 7, nz - 1, nz, nz + 5, R, R + 9):
        budget = cap * 256 + 255                              # floor division by bytes_per_row
        rc, st, sel = oracle.plan_replication(None, None, 1, 1, None, R, counts.copy(), S, budget, 256)
        assert rc == 0 and st == 0
        assert np.array_equal(sel, order[:min(cap, nz)])
        rc, st, sel = oracle.plan_replication(None, None, 1, 1, None, R, counts.copy(), S | Z, budget, 256)
        assert np.array_equal(sel, order[:min(cap, R)])


def test_select_closed_forms():
    # all counts equal: the tie-break alone decides -> rows 0 .. k-1
    counts = np.full(50, 9, np.uint32)
    assert oracle.plan_replication(None, None, 1, 1, None, 50, counts, S, 20 * 8, 8)[2].tolist() == list(range(20))
    # counts exactly proportional to a Zipf pmf through a permutation: selection = the permutation's head
    rng = np.random.default_rng(8)
    E, k = 300, 40
    perm = rng.permutation(E)
    counts = np.zeros(E, np.uint32)
    counts[perm] = np.floor(1e6 * np.arange(1, E + 1, dtype=np.float64) ** -1.3).astype(np.uint32) + (E - np.arange(E))
    assert np.array_equal(oracle.plan_replication(None, None, 1, 1, None, E, counts, S, k, 1)[2], perm[:k])
    # merged tables (Section 4.6): one global order, table index is the major tie-break key
    counts = np.array([5, 1, 5, 0, 7, 5], np.uint32)          # two tables of 3 rows
    assert oracle.plan_replication(None, None, 1, 1, None, 6, counts, S, 4, 1)[2].tolist() == [4, 0, 2, 5]


def test_tagging_and_end_to_end():
    rng = np.random.default_rng(2)
    T, B, E = 2, 6, 20
    ids, offsets, row_base, n = random_jagged(rng, T, B, E, 25)
    counts = np.zeros(T * E, np.uint32)
    placement = np.array([entry(2, r % 4) for r in range(T * E)], np.uint32)
    rc, st, sel = oracle.plan_replication(ids, offsets, T, B, row_base, T * E, counts, A | S | TAG, 5 * 64, 64, placement)
    assert rc == 0 and len(sel) == 5
    assert np.all(placement[sel] >> 30 == 0) and np.all(placement[sel] & 0x3FFFFFFF == sel % 4)
    rest = np.setdiff1d(np.arange(T * E), sel)
    assert np.all(placement[rest] >> 30 == 2)
    # routing after tagging: the selected rows are served locally (Section 3.1, data-parallel rows)
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(ids, offsets, T, B, row_base, placement, 4, 2, 3)
    g = row_base[table_of(offsets, B)] + ids
    assert tc[0] == np.isin(g, sel).sum() and set(np.nonzero(np.isin(g, sel))[0]) <= set(pos[bo[3]:bo[4]].tolist())


def test_plan_host_faults():
    c = np.zeros(4, np.uint32)
    assert oracle.plan_replication(None, None, 1, 1, None, 4, c, 16)[0] == 6
    assert oracle.plan_replication(None, None, 1, 1, None, 4, c, TAG)[0] == 6
    assert oracle.plan_replication(None, None, 1, 1, None, 4, c, S, -1, 1)[0] == 2
    assert oracle.plan_replication(None, None, 1, 1, None, 4, c, S, 1, 0)[0] == 2
    assert oracle.plan_replication(None, None, 1, 1, None, 4, c, S | TAG, 1, 1)[0] == 1
    assert oracle.plan_replication(None, None, 1, 1, None, 4, c, 0)[0] == 0


# ------------------------------------------------------------------ what the paper prints
def test_paper_tier_sizes_partition_the_table():
    """Every row is in exactly one tier: the printed tier sizes sum to the table size, and a
    placement built with those sizes (scaled by the 32 GPUs they are all multiples of) routes a
    sweep over all rows into exactly those tier counts."""
    G = golden()
    assert G["rm1_2tier_dp"] + G["rm1_2tier_rw"] == G["rm1_rows"]
    assert G["rm1_3tier_dp"] + G["rm1_3tier_flex"] + G["rm1_3tier_rw"] == G["rm1_rows"]
    assert G["rm2_3tier_dp"] + G["rm2_3tier_flex"] + G["rm2_3tier_rw"] == G["rm1_rows"]
    assert G["rm3_3tier_dp"] + G["rm3_3tier_flex"] + G["rm3_3tier_rw"] == G["rm3_rows"]
    assert G["rm4_3tier_dp"] + G["rm4_3tier_flex"] + G["rm4_3tier_rw"] == G["rm3_rows"]
    dp, fx, rw = (G[k] // 32 for k in ("rm3_3tier_dp", "rm3_3tier_flex", "rm3_3tier_rw"))
    E = dp + fx + rw
    rng = np.random.default_rng(0)
    perm = rng.permutation(E)
    placement = np.empty(E, np.uint32)
    placement[perm[:dp]] = entry(0)
    placement[perm[dp:dp + fx]] = (1 << 30) | (perm[dp:dp + fx] % 8)
    placement[perm[dp + fx:]] = (2 << 30) | (perm[dp + fx:] % 32)
    rc, st, bo, rows, pos, tc = oracle.route_bucketize(np.arange(E), [0, E], 1, 1, [0, E], placement, 32, 8, 9)
    assert rc == 0 and st == 0 and tc.tolist() == [dp, fx, rw]
    # lookups that stay inside the requester's group: tiers 0 and 1, plus the sharded rows it owns
    own = perm[dp + fx:] % 32
    assert bo[16] - bo[8] == dp + fx + int(((own >= 8) & (own < 16)).sum())


def test_paper_activation_size():
    """The sequence output holds every looked-up row: batch x length x D x 4 bytes."""
    G = golden()
    n = G["rm1_local_batch"] * G["rm1_avg_length"]
    assert round(n * G["rm1_dim"] * 4 / 1e9, 2) == G["rm1_activation_gb"]
    assert round(G["rm1_local_batch"] * G["rm3_avg_length"] * G["rm1_dim"] * 4 / 1e9, 2) == G["rm3_activation_gb"]
    # and the oracle's gather writes exactly one D-row per lookup (scaled down 1/4096)
    W = np.ones((10, 256), np.float32)
    out = np.zeros((1000, 256), np.float32)
    oracle.seq_gather_fwd(W, np.zeros(1000, np.int64), np.arange(1000, dtype=np.int32), 0, 1000, out)
    assert out.nbytes * 4096 == n * G["rm1_dim"] * 4 and out.sum() == 1000 * 256


def test_paper_a2a_reduction_is_share_of_local_lookups():
    G = golden()
    assert round(100 * (1 - G["rm2_a2a_3tier_bytes"] / G["rm2_a2a_rw_bytes"]), 1) == G["rm2_a2a_3tier_reduction_pct"]
    assert round(100 * (1 - G["rm1_a2a_2tier_bytes"] / G["rm1_a2a_rw_bytes"]), 1) == G["rm1_a2a_2tier_reduction_pct"]
