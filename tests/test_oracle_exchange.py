"""Pins for the oracle's two halves of the row exchange and its replica store.

Section 3.2 (metric 2, "dynamic communication"): the owner sends the looked-up rows back in the
order the ids arrived, the requester puts them where the lookups were.  The owner half is
numpy.take, the requester half is a fancy-index assignment (numpy.put along rows), and the two
in a row must write what the one-step gather writes.  The replica store (Section 3.1: a
replicated row is served locally; Section 4.3: the popular rows are the replicated ones) is
numpy.take of the selected rows plus a first-occurrence map found by brute force.
"""
import numpy as np
import pytest

import oracle
from helpers import bf16_bits_from_f32


def _table(rng, R, D, dt):
    if dt == "f32":
        return rng.standard_normal((R, D)).astype(np.float32), oracle.F32
    if dt == "f16":
        return rng.standard_normal((R, D)).astype(np.float16), oracle.F16
    return bf16_bits_from_f32(rng.standard_normal((R, D))), oracle.BF16


@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
def test_send_is_take_and_unbucketize_is_row_assignment(dt):
    rng = np.random.default_rng(11)
    R, D, n = 150, {"f32": 4, "f16": 16, "bf16": 24}[dt], 401
    W, code = _table(rng, R, D, dt)
    g = rng.integers(0, R, n)
    perm = rng.permutation(n).astype(np.int32)
    rows = g[perm]
    j0, j1 = 37, 300
    send = np.full((j1 - j0, D), 9, W.dtype)
    assert oracle.seq_gather_send(W, rows, j0, j1, send, dtype=code) == (0, 0)
    assert np.array_equal(send.view(np.uint8), np.take(W, rows[j0:j1], axis=0).view(np.uint8))
    out = np.full((n, D), 5, W.dtype)
    assert oracle.seq_unbucketize(send, perm, j0, j1, out, dtype=code) == (0, 0)
    expect = np.full((n, D), 5, W.dtype)
    expect[perm[j0:j1]] = send                      # positions are distinct: a plain row assignment
    assert np.array_equal(out.view(np.uint8), expect.view(np.uint8))
    # the two halves in a row = the one-step gather over the same range
    direct = np.full((n, D), 5, W.dtype)
    assert oracle.seq_gather_fwd(W, rows, perm, j0, j1, direct, dtype=code) == (0, 0)
    assert np.array_equal(out.view(np.uint8), direct.view(np.uint8))


def test_send_and_unbucketize_do_not_mix_up_their_indices():
    # asymmetric sizes: a send indexed by position or an unbucketize indexed by row would leave the arrays
    W = np.arange(6 * 4, dtype=np.float32).reshape(6, 4)
    rows = np.array([5, 0, 3], np.int64)
    pos = np.array([1, 2, 0], np.int32)
    send = np.zeros((2, 4), np.float32)
    assert oracle.seq_gather_send(W, rows, 1, 3, send) == (0, 0)
    assert send.tolist() == [W[0].tolist(), W[3].tolist()]
    out = np.full((3, 4), -1, np.float32)
    assert oracle.seq_unbucketize(send, pos, 1, 3, out) == (0, 0)
    assert out.tolist() == [W[3].tolist(), [-1.0] * 4, W[0].tolist()]


def test_exchange_faults():
    W = np.arange(8 * 4, dtype=np.float32).reshape(8, 4)
    send = np.full((4, 4), -1, np.float32)
    rc, st = oracle.seq_gather_send(W, [1, 8, -1, 2], 0, 4, send)
    assert (rc, st) == (0, oracle.BAD_ID)
    assert np.array_equal(send[0], W[1]) and np.all(send[1:3] == -1) and np.array_equal(send[3], W[2])
    out = np.full((3, 4), -1, np.float32)
    rc, st = oracle.seq_unbucketize(send, np.array([2, 3, -1, 0], np.int32), 0, 4, out)
    assert (rc, st) == (0, oracle.BAD_ID)
    assert np.array_equal(out[2], W[1]) and np.all(out[1] == -1) and np.array_equal(out[0], W[2])
    assert oracle.seq_gather_send(W, [0], 1, 0, send)[0] == 2
    assert oracle.seq_unbucketize(send, np.array([0], np.int32), 1, 0, out)[0] == 2
    assert oracle.seq_gather_send(W[:, :3].copy(), [0], 0, 1, send[:, :3].copy())[0] == 4
    assert oracle.seq_gather_send(W, [0], 0, 0, send) == (0, 0)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_replica_store_is_take_with_first_occurrence_map(dt):
    rng = np.random.default_rng(5)
    R, D = 90, 8
    W, code = _table(rng, R, D, dt)
    sel = rng.permutation(R)[:20].astype(np.int64)
    sel[7] = sel[2]                                   # a duplicate: the first slot wins
    store = np.zeros((20, D), W.dtype)
    rc, st, slots = oracle.replica_build(W, sel, store, dtype=code)
    assert (rc, st) == (0, 0)
    assert np.array_equal(store.view(np.uint8), np.take(W, sel, axis=0).view(np.uint8))
    brute = np.full(R, -1, np.int32)
    for r in range(R):
        for s in range(len(sel)):
            if sel[s] == r:
                brute[r] = s
                break
    assert np.array_equal(slots, brute) and slots[sel[2]] == 2
    # gather through the store = plain gather; prove the store is really read by changing it
    n = 300
    g = rng.integers(0, R, n)
    perm = rng.permutation(n).astype(np.int32)
    out = np.zeros((n, D), W.dtype)
    assert oracle.seq_gather_fwd_replica(W, store, slots, g[perm], perm, 0, n, out, dtype=code) == (0, 0)
    assert np.array_equal(out.view(np.uint8), np.take(W, g, axis=0).view(np.uint8))
    marked = store.copy()
    marked[:] = 0
    out2 = np.full((n, D), 1, W.dtype)
    assert oracle.seq_gather_fwd_replica(W, marked, slots, g[perm], perm, 0, n, out2, dtype=code) == (0, 0)
    in_store = slots[g] >= 0
    assert in_store.any() and (~in_store).any()
    assert np.all(out2[in_store] == 0)
    assert np.array_equal(out2[~in_store].view(np.uint8), np.take(W, g[~in_store], axis=0).view(np.uint8))


def test_replica_faults_and_empty():
    W = np.arange(8 * 4, dtype=np.float32).reshape(8, 4)
    store = np.full((3, 4), -1, np.float32)
    rc, st, slots = oracle.replica_build(W, [4, 8, 1], store)
    assert (rc, st) == (0, oracle.BAD_ID)
    assert slots.tolist() == [-1, 2, -1, -1, 0, -1, -1, -1]
    assert np.array_equal(store[0], W[4]) and np.all(store[1] == -1) and np.array_equal(store[2], W[1])
    rc, st, slots0 = oracle.replica_build(W, [], np.zeros((0, 4), np.float32))
    assert (rc, st) == (0, 0) and np.all(slots0 == -1)
    # a slot beyond the store is a data fault and skips the lookup
    bad = slots.copy()
    bad[1] = 3
    out = np.full((2, 4), -1, np.float32)
    rc, st = oracle.seq_gather_fwd_replica(W, store, bad, [1, 4], np.array([0, 1], np.int32), 0, 2, out)
    assert (rc, st) == (0, oracle.BAD_ID) and np.all(out[0] == -1) and np.array_equal(out[1], W[4])


def test_slots_travel_in_the_placement_of_replicated_rows():
    """The slot hand-over: a tier-0 entry's owner bits become the row's slot (NO_SLOT without one), other tiers
    stay as they are; reading a lookup's slot back is a take through the tagged placement; and the gather with
    the slots given writes what the gather with the slot map writes -- which, with a store built from the same
    table, is numpy.take."""
    from helpers import entry, random_placement
    rng = np.random.default_rng(5)
    R, D, k, n = 400, 8, 37, 900
    W, code = _table(rng, R, D, "f32")
    pl = random_placement(rng, R, 8, 4, p=(0.5, 0.2, 0.3))
    before = pl.copy()
    sel = np.concatenate([rng.permutation(R)[:k - 2], [-3, R + 9]]).astype(np.int64)     # two faulty selections
    store = np.zeros((k, D), np.float32)
    rc, st, slot_of_row = oracle.replica_build(W, sel, store)
    assert rc == 0 and st == oracle.BAD_ID
    assert oracle.replica_tag_slots(pl, slot_of_row) == (0, 0)
    tier = before >> 30
    assert np.array_equal(pl[tier != 0], before[tier != 0])                              # other tiers untouched
    want = np.where(slot_of_row >= 0, slot_of_row, oracle.NO_SLOT).astype(np.uint32)
    assert np.array_equal(pl[tier == 0], want[tier == 0]) and np.all(pl[tier == 0] >> 30 == 0)
    # a lookup's slot: its row's, if the row is replicated here and has one
    rows = rng.integers(0, R, n)
    rows[:5] = sel[:5]
    rc, st, got = oracle.lookup_slots(pl, rows, 100, 850)
    exp = np.where((tier[rows] == 0) & (slot_of_row[rows] >= 0), slot_of_row[rows], -1)
    assert (rc, st) == (0, 0) and np.array_equal(got[100:850], exp[100:850]) and np.all(got[:100] == -7) and np.all(got[850:] == -7)
    rc, st, all_slots = oracle.lookup_slots(pl, rows, 0, n)
    # the gather with slots: a marked store tells where each row came from
    pos = rng.permutation(n).astype(np.int32)
    mark = store + 1000.0
    out = np.zeros((n, D), np.float32)
    assert oracle.seq_gather_fwd_slots(W, mark, rows, all_slots, pos, 0, n, out) == (0, 0)
    ref = np.zeros((n, D), np.float32)
    ref[pos] = np.where((all_slots >= 0)[:, None], mark[np.maximum(all_slots, 0)], W[rows])
    assert np.array_equal(out, ref) and (all_slots >= 0).sum() > 20
    # with the store the table's own rows: the plain lookup, bit for bit, also over a sub-range
    out2 = np.full((n, D), 5.0, np.float32)
    assert oracle.seq_gather_fwd_slots(W, store, rows, all_slots, pos, 200, 700, out2) == (0, 0)
    ref2 = np.full((n, D), 5.0, np.float32)
    ref2[pos[200:700]] = W[rows[200:700]]
    assert np.array_equal(out2, ref2)


def test_slot_faults():
    from helpers import entry
    W = np.arange(40, dtype=np.float32).reshape(10, 4)
    store = W[:3] + 100
    # a slot number that the owner bits cannot hold, a row outside the table, a slot beyond the store
    pl = np.array([entry(0, 7), entry(0, 7), entry(2, 1)], np.uint32)
    assert oracle.replica_tag_slots(pl, [oracle.NO_SLOT, 2, 0]) == (0, oracle.BAD_ID)
    assert pl.tolist() == [oracle.NO_SLOT, 2, entry(2, 1)]
    rc, st, s = oracle.lookup_slots(pl, [1, 3, -1, 0, 2], 0, 5)
    assert (rc, st) == (0, oracle.BAD_ID) and s.tolist() == [2, -1, -1, -1, -1]
    out = np.zeros((4, 4), np.float32)
    rc, st = oracle.seq_gather_fwd_slots(W, store, [4, 5, 6, 11], [1, 3, -1, 0], np.array([0, 1, 2, 3], np.int32), 0, 4, out)
    assert (rc, st) == (0, oracle.BAD_ID)
    assert np.array_equal(out, np.stack([store[1], np.zeros(4), W[6], np.zeros(4)]).astype(np.float32))
    assert oracle.replica_tag_slots(pl, [0, 0, 0])[0] == 0 and oracle.lookup_slots(pl, [0], 1, 0)[0] == 2
