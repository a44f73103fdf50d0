"""GPU parity: fs_seq_gather_send, fs_seq_unbucketize, fs_replica_build and
fs_seq_gather_fwd_replica against the CPU oracle, bit for bit, and the compositions that must
reproduce fs_seq_gather_fwd."""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def _status(G):
    return torch.zeros(1, dtype=torch.int32, device=G.DEV)


@pytest.mark.parametrize("dt,D", [("f32", 4), ("f16", 8), ("f32", 64), ("bf16", 128), ("bf16", 256), ("f16", 24),
                                  ("f32", 520)])
def test_send_and_unbucketize_bit_exact(G, dt, D):
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(D + 1)
    tdt = TDT[dt]
    R, n = 3000, 5003
    Wt = torch.randn(R, D, generator=torch.Generator().manual_seed(D)).to(tdt)
    g = rng.integers(0, R, n)
    perm = rng.permutation(n).astype(np.int32)
    rows = g[perm]
    rows_d, pos_d, W_d = G.to_dev(rows, torch.int64), G.to_dev(perm, torch.int32), Wt.to(G.DEV)
    Wn = fs_inputs.as_numpy_bits(Wt)
    code = G.oracle_dtype(dt)
    for j0, j1 in ((0, n), (777, 4099)):
        m = j1 - j0
        st = _status(G)
        send = torch.full((m, D), 3.0, dtype=tdt, device=G.DEV)
        assert fs.fs_seq_gather_send(W_d, rows_d, j0, j1, send, st) == 0
        ref_send = fs_inputs.as_numpy_bits(torch.full((m, D), 3.0, dtype=tdt)).copy()
        assert oracle.seq_gather_send(Wn, rows, j0, j1, ref_send, dtype=code) == (0, 0)
        assert np.array_equal(G.bits(send), ref_send.view(np.uint8).reshape(-1))
        out = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
        assert fs.fs_seq_unbucketize(send, pos_d, j0, j1, out, st) == 0
        ref_out = fs_inputs.as_numpy_bits(torch.full((n, D), 7.0, dtype=tdt)).copy()
        assert oracle.seq_unbucketize(ref_send, perm, j0, j1, ref_out, dtype=code) == (0, 0)
        assert np.array_equal(G.bits(out), ref_out.view(np.uint8).reshape(-1))
        # the two halves in a row write what the one-step gather writes
        direct = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
        assert fs.fs_seq_gather_fwd(W_d, rows_d, pos_d, j0, j1, direct, st) == 0
        torch.cuda.synchronize()
        assert int(st.item()) == 0 and torch.equal(out.view(torch.uint8), direct.view(torch.uint8))


def test_exchange_faults(G):
    import paper_2301_02959_amd as fs
    Wt = torch.arange(8 * 4, dtype=torch.float32).reshape(8, 4).to(G.DEV)
    st = _status(G)
    send = torch.full((4, 4), -1.0, device=G.DEV)
    rows = G.to_dev([1, 8, -1, 2], torch.int64)
    assert fs.fs_seq_gather_send(Wt, rows, 0, 4, send, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID
    assert torch.equal(send[0], Wt[1]) and torch.all(send[1:3] == -1) and torch.equal(send[3], Wt[2])
    st.zero_()
    out = torch.full((3, 4), -1.0, device=G.DEV)
    pos = G.to_dev([2, 3, -1, 0], torch.int32)
    assert fs.fs_seq_unbucketize(send, pos, 0, 4, out, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID
    assert torch.equal(out[2], Wt[1]) and torch.all(out[1] == -1) and torch.equal(out[0], Wt[2])
    # host faults
    assert fs.fs_seq_gather_send(Wt, rows, 2, 2, send, st) == 0
    assert fs.fs_seq_gather_send(Wt, rows, 3, 2, send, st, raise_on_error=False) == 2
    assert fs.fs_seq_gather_send(Wt, None, 0, 1, send, st, raise_on_error=False) == 1
    assert fs.fs_seq_gather_send(Wt, rows, 0, 1, send, st, raise_on_error=False, D=3) == 4
    assert fs.fs_seq_gather_send(Wt, rows, 0, 1, send, st, raise_on_error=False, dtype=9) == 3
    assert fs.fs_seq_unbucketize(send, pos, 2, 2, out, st) == 0
    assert fs.fs_seq_unbucketize(send, pos, 3, 2, out, st, raise_on_error=False) == 2
    assert fs.fs_seq_unbucketize(send, None, 0, 1, out, st, raise_on_error=False) == 1
    assert fs.fs_seq_unbucketize(send, pos, 0, 1, out, st, raise_on_error=False, D=2) == 4
    assert fs.fs_seq_unbucketize(send, pos, 0, 1, out, st, raise_on_error=False, n=1 << 31) == 2
    torch.cuda.synchronize()


@pytest.mark.parametrize("dt,D", [("f32", 8), ("bf16", 256), ("f16", 72)])
def test_replica_build_and_gather_bit_exact(G, dt, D):
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(D + 2)
    tdt = TDT[dt]
    R, n, k = 4000, 6007, 700
    Wt = torch.randn(R, D, generator=torch.Generator().manual_seed(D)).to(tdt)
    Wn = fs_inputs.as_numpy_bits(Wt)
    code = G.oracle_dtype(dt)
    sel = rng.permutation(R)[:k].astype(np.int64)
    sel[100] = sel[5]                                   # duplicate: first slot wins
    W_d, sel_d = Wt.to(G.DEV), G.to_dev(sel, torch.int64)
    st = _status(G)
    for k_dev in (None, k, 333, 0):                     # device-side count: absent, full, shorter, empty
        k_eff = k if k_dev is None else k_dev
        store = torch.full((k, D), 2.0, dtype=tdt, device=G.DEV)
        slots = torch.full((R,), 12345, dtype=torch.int32, device=G.DEV)
        nsel = None if k_dev is None else torch.tensor([k_dev], dtype=torch.int64, device=G.DEV)
        assert fs.fs_replica_build(W_d, sel_d, k, nsel, store, slots, st) == 0
        ref_store = fs_inputs.as_numpy_bits(torch.full((k, D), 2.0, dtype=tdt)).copy()
        rc, ost, ref_slots = oracle.replica_build(Wn, sel[:k_eff], ref_store[:k_eff], dtype=code)
        torch.cuda.synchronize()
        assert (rc, ost) == (0, 0) and int(st.item()) == 0
        assert np.array_equal(slots.cpu().numpy(), ref_slots)
        assert np.array_equal(G.bits(store), ref_store.view(np.uint8).reshape(-1))
        # lookups: half of them aimed at the replicated rows
        g = np.where(rng.random(n) < 0.5, sel[rng.integers(0, k, n)], rng.integers(0, R, n))
        perm = rng.permutation(n).astype(np.int32)
        rows_d, pos_d = G.to_dev(g[perm], torch.int64), G.to_dev(perm, torch.int32)
        out = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
        assert fs.fs_seq_gather_fwd_replica(W_d, store, k, slots, rows_d, pos_d, 0, n, out, st) == 0
        ref = fs_inputs.as_numpy_bits(torch.full((n, D), 7.0, dtype=tdt)).copy()
        assert oracle.seq_gather_fwd_replica(Wn, ref_store, ref_slots, g[perm], perm, 0, n, ref, dtype=code) == (0, 0)
        direct = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
        assert fs.fs_seq_gather_fwd(W_d, rows_d, pos_d, 0, n, direct, st) == 0
        torch.cuda.synchronize()
        assert int(st.item()) == 0
        assert np.array_equal(G.bits(out), ref.view(np.uint8).reshape(-1))
        assert torch.equal(out.view(torch.uint8), direct.view(torch.uint8))
        # the store is what is read: change it and the replicated lookups change with it
        store.zero_()
        out2 = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
        assert fs.fs_seq_gather_fwd_replica(W_d, store, k, slots, rows_d, pos_d, 100, n - 100, out2, st) == 0
        ref2 = fs_inputs.as_numpy_bits(torch.full((n, D), 7.0, dtype=tdt)).copy()
        ref_zero = np.zeros_like(ref_store)
        oracle.seq_gather_fwd_replica(Wn, ref_zero, ref_slots, g[perm], perm, 100, n - 100, ref2, dtype=code)
        torch.cuda.synchronize()
        assert np.array_equal(G.bits(out2), ref2.view(np.uint8).reshape(-1))


def test_replica_faults(G):
    import paper_2301_02959_amd as fs
    Wt = torch.arange(8 * 4, dtype=torch.float32).reshape(8, 4).to(G.DEV)
    st = _status(G)
    store = torch.full((3, 4), -1.0, device=G.DEV)
    slots = torch.zeros(8, dtype=torch.int32, device=G.DEV)
    sel = G.to_dev([4, 8, 1], torch.int64)
    assert fs.fs_replica_build(Wt, sel, 3, None, store, slots, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID
    assert slots.tolist() == [-1, 2, -1, -1, 0, -1, -1, -1]
    assert torch.equal(store[0], Wt[4]) and torch.all(store[1] == -1) and torch.equal(store[2], Wt[1])
    # a slot beyond the store skips the lookup
    st.zero_()
    bad = slots.clone()
    bad[1] = 3
    out = torch.full((2, 4), -1.0, device=G.DEV)
    rows, pos = G.to_dev([1, 4], torch.int64), G.to_dev([0, 1], torch.int32)
    assert fs.fs_seq_gather_fwd_replica(Wt, store, 3, bad, rows, pos, 0, 2, out, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID and torch.all(out[0] == -1) and torch.equal(out[1], Wt[4])
    # k = 0: every slot -1, the gather reads the table only
    assert fs.fs_replica_build(Wt, None, 0, None, None, slots, st) == 0
    torch.cuda.synchronize()
    assert torch.all(slots == -1)
    assert fs.fs_seq_gather_fwd_replica(Wt, None, 0, slots, rows, pos, 0, 2, out, st) == 0
    torch.cuda.synchronize()
    assert torch.equal(out[0], Wt[1]) and torch.equal(out[1], Wt[4])
    # host faults
    assert fs.fs_replica_build(Wt, sel, -1, None, store, slots, st, raise_on_error=False) == 2
    assert fs.fs_replica_build(Wt, None, 3, None, store, slots, st, raise_on_error=False) == 1
    assert fs.fs_replica_build(Wt, sel, 3, None, store, None, st, raise_on_error=False) == 1
    assert fs.fs_replica_build(Wt, sel, 3, None, store, slots, st, raise_on_error=False, D=3) == 4
    assert fs.fs_seq_gather_fwd_replica(Wt, store, 3, None, rows, pos, 0, 2, out, st, raise_on_error=False) == 1
    assert fs.fs_seq_gather_fwd_replica(Wt, store, -1, slots, rows, pos, 0, 2, out, st, raise_on_error=False) == 2
    torch.cuda.synchronize()


def test_c1_plan_replica_route_exchange_end_to_end(G):
    """plan -> replica store -> route -> per-bucket send / unbucketize with the own bucket served
    through the store: the assembled output is the plain lookup."""
    import paper_2301_02959_amd as fs
    cfg = fs_inputs.CONFIGS["c1"]
    b, pl = G.batch_on(cfg, G.DEV)
    Wt = fs_inputs.make_table(cfg).to(G.DEV)
    n, R = b["n"], cfg.R
    counts = torch.zeros(R, dtype=torch.int32, device=G.DEV)
    k_cap = 64
    sel = torch.full((k_cap,), -1, dtype=torch.int64, device=G.DEV)
    nsel = torch.zeros(1, dtype=torch.int64, device=G.DEV)
    st = _status(G)
    row_bytes = cfg.D * 4
    fs.fs_plan_replication(b["ids"], b["offsets"], cfg.T, cfg.B, b["row_base"], n, R, counts,
                           fs.FS_PLAN_ACCUMULATE | fs.FS_PLAN_SELECT | fs.FS_PLAN_TAG, k_cap * row_bytes, row_bytes,
                           sel, nsel, pl, st)
    store = torch.zeros(k_cap, cfg.D, device=G.DEV)
    slots = torch.zeros(R, dtype=torch.int32, device=G.DEV)
    fs.fs_replica_build(Wt, sel, k_cap, nsel, store, slots, st)
    self_ = 3
    rc, rst, bo, rows, pos, tc = G.hip_route(b["ids"], b["offsets"], cfg.T, cfg.B, b["row_base"], pl, cfg.U, cfg.W, self_)
    bo = bo.cpu().tolist()
    out = torch.full((n, cfg.D), float("nan"), device=G.DEV)
    for u in range(cfg.U):
        lo, hi = bo[u], bo[u + 1]
        if u == self_:
            fs.fs_seq_gather_fwd_replica(Wt, store, k_cap, slots, rows, pos, lo, hi, out, st)
        else:
            send = torch.empty(hi - lo, cfg.D, device=G.DEV)
            fs.fs_seq_gather_send(Wt, rows, lo, hi, send, st)
            fs.fs_seq_unbucketize(send, pos, lo, hi, out, st)
    torch.cuda.synchronize()
    assert int(st.item()) == 0 and int(tc[0]) > 0
    assert torch.equal(out, Wt[b["ids"]])


@pytest.mark.parametrize("dt,D,U,W", [("f32", 8, 8, 4), ("bf16", 256, 64, 8), ("f16", 72, 24, 24)])
def test_slots_from_the_router_bit_exact(G, dt, D, U, W):
    """The slot hand-over: fs_replica_tag_slots writes what the oracle writes into the placement;
    fs_route_bucketize_slots gives fs_route_bucketize's outputs plus the oracle's slot of every lookup;
    fs_seq_gather_fwd_slots with those slots writes the oracle's bits, which are the plain gather's when the
    store holds the table's own rows, and the store's when it does not."""
    import paper_2301_02959_amd as fs
    from helpers import random_jagged, random_placement
    rng = np.random.default_rng(D + U)
    tdt = TDT[dt]
    code = G.oracle_dtype(dt)
    T, B, E, k = 3, 40, 5000, 900
    R = T * E
    ids, offsets, row_base, n = random_jagged(rng, T, B, E, 200)
    ids = np.minimum(rng.pareto(0.9, n).astype(np.int64) * 3, E - 1)            # skewed: the popular rows repeat
    pl = random_placement(rng, R, U, W, p=(0.4, 0.2, 0.4))
    Wt = torch.randn(R, D, generator=torch.Generator().manual_seed(D)).to(tdt)
    Wn = fs_inputs.as_numpy_bits(Wt)
    # the store: the k most looked-up rows, whatever their tier (only tier-0 rows will be served from it)
    g_all = row_base[np.repeat(np.arange(T * B), np.diff(offsets)) // B] + ids
    sel = np.argsort(-np.bincount(g_all, minlength=R), kind="stable")[:k].astype(np.int64)
    W_d, sel_d, pl_d = Wt.to(G.DEV), G.to_dev(sel, torch.int64), G.placement_dev(pl)
    st = _status(G)
    store = torch.zeros(k, D, dtype=tdt, device=G.DEV)
    slot_of_row = torch.zeros(R, dtype=torch.int32, device=G.DEV)
    assert fs.fs_replica_build(W_d, sel_d, k, None, store, slot_of_row, st) == 0
    assert fs.fs_replica_tag_slots(pl_d, slot_of_row, st) == 0
    ref_store = np.zeros_like(Wn[:k])
    rc, ost, ref_slot_of_row = oracle.replica_build(Wn, sel, ref_store, dtype=code)
    pl_tagged = pl.copy()
    assert oracle.replica_tag_slots(pl_tagged, ref_slot_of_row) == (0, 0)
    torch.cuda.synchronize()
    assert int(st.item()) == 0 and np.array_equal(pl_d.cpu().numpy().view(np.uint32), pl_tagged)
    # the router
    self_ = U - 1
    ids_d, off_d, rb_d = G.to_dev(ids, torch.int64), G.to_dev(offsets, torch.int64), G.to_dev(row_base, torch.int64)
    bo = torch.zeros(U + 1, dtype=torch.int64, device=G.DEV)
    rows = torch.zeros(n, dtype=torch.int64, device=G.DEV)
    pos = torch.zeros(n, dtype=torch.int32, device=G.DEV)
    slots = torch.full((n,), -7, dtype=torch.int32, device=G.DEV)
    tc = torch.zeros(3, dtype=torch.int64, device=G.DEV)
    assert fs.fs_route_bucketize_slots(ids_d, off_d, T, B, rb_d, pl_d, n, U, W, self_, bo, rows, pos, slots, tc, st) == 0
    orc, ost, obo, orows, opos, otc = oracle.route_bucketize(ids, offsets, T, B, row_base, pl_tagged, U, W, self_)
    rc2, st2, oslots = oracle.lookup_slots(pl_tagged, orows, 0, n)
    torch.cuda.synchronize()
    assert (orc, ost, rc2, st2) == (0, 0, 0, 0) and int(st.item()) == 0
    assert np.array_equal(bo.cpu().numpy(), obo) and np.array_equal(tc.cpu().numpy(), otc)
    assert np.array_equal(rows.cpu().numpy(), orows) and np.array_equal(pos.cpu().numpy(), opos)
    assert np.array_equal(slots.cpu().numpy(), oslots) and (oslots >= 0).sum() > n // 10
    # the gather that takes the slots: a marked store shows which lookups it served
    mark = (store.float() + 1000.0).to(tdt)
    mark_n = fs_inputs.as_numpy_bits(mark)
    for j0, j1, src_d, src_n in ((0, n, mark, mark_n), (n // 7, n - 5, store, ref_store)):
        out = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
        assert fs.fs_seq_gather_fwd_slots(W_d, src_d, k, rows, slots, pos, j0, j1, out, st) == 0
        ref = fs_inputs.as_numpy_bits(torch.full((n, D), 7.0, dtype=tdt)).copy()
        assert oracle.seq_gather_fwd_slots(Wn, src_n, orows, oslots, opos, j0, j1, ref, dtype=code) == (0, 0)
        torch.cuda.synchronize()
        assert int(st.item()) == 0 and np.array_equal(G.bits(out), ref.view(np.uint8).reshape(-1))
    direct = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
    assert fs.fs_seq_gather_fwd(W_d, rows, pos, n // 7, n - 5, direct, st) == 0
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.uint8), direct.view(torch.uint8))       # the store's rows are the table's


def test_slot_faults(G):
    import paper_2301_02959_amd as fs
    from helpers import entry
    Wt = torch.arange(10 * 4, dtype=torch.float32).reshape(10, 4).to(G.DEV)
    store = Wt[:3] + 100
    st = _status(G)
    # a slot number that the owner bits cannot hold; entries of other tiers stay
    pl = G.placement_dev(np.array([entry(0, 7), entry(0, 7), entry(2, 1)], np.uint32))
    assert fs.fs_replica_tag_slots(pl, G.to_dev([oracle.NO_SLOT, 2, 0], torch.int32), st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID and pl.cpu().numpy().view(np.uint32).tolist() == [oracle.NO_SLOT, 2, entry(2, 1)]
    # a slot beyond the store and a row outside the table skip the lookup
    st.zero_()
    out = torch.zeros(4, 4, device=G.DEV)
    rows, slots, pos = G.to_dev([4, 5, 6, 11], torch.int64), G.to_dev([1, 3, -1, 0], torch.int32), G.to_dev([0, 1, 2, 3], torch.int32)
    assert fs.fs_seq_gather_fwd_slots(Wt, store, 3, rows, slots, pos, 0, 4, out, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID
    assert torch.equal(out, torch.stack([store[1], torch.zeros(4, device=G.DEV), Wt[6], torch.zeros(4, device=G.DEV)]))
    # host faults
    assert fs.fs_replica_tag_slots(None, slots, st, raise_on_error=False, R=3) == 1
    assert fs.fs_replica_tag_slots(pl, slots, st, raise_on_error=False, R=0) == 2
    assert fs.fs_seq_gather_fwd_slots(Wt, store, 3, rows, None, pos, 0, 4, out, st, raise_on_error=False) == 1
    assert fs.fs_seq_gather_fwd_slots(Wt, store, -1, rows, slots, pos, 0, 4, out, st, raise_on_error=False) == 2
    assert fs.fs_seq_gather_fwd_slots(Wt, store, 3, rows, slots, pos, 3, 2, out, st, raise_on_error=False) == 2
    z64 = torch.zeros(4, dtype=torch.int64, device=G.DEV)
    off = G.to_dev([0, 4], torch.int64)
    rb = G.to_dev([0, 3], torch.int64)
    bo = torch.zeros(2, dtype=torch.int64, device=G.DEV)
    assert fs.fs_route_bucketize_slots(z64, off, 1, 1, rb, pl, 4, 1, 1, 0, bo, z64.clone(), pos.clone(), None, None, st,
                                       raise_on_error=False) == 1
    # an empty batch: offsets written, nothing else
    off0 = G.to_dev([0, 0], torch.int64)
    assert fs.fs_route_bucketize_slots(None, off0, 1, 1, rb, pl, 0, 1, 1, 0, bo, None, None, None, None, st) == 0
    torch.cuda.synchronize()
    assert bo.tolist() == [0, 0]
