"""The largest batch the interface admits, n = 2^31 - 1 lookups, through route + bucketize, gather
and backward on one GPU: every index that could overflow 32 bits does so here if it is going to.

The oracle cannot walk 2.1 billion lookups in test time, so the results are checked through
properties that determine them completely:
  route     bucket_offsets = running sum of the destinations' bincount; inside a bucket the positions
            ascend; every (row, position) pair is a lookup of the batch with that destination
            (together: the stable counting sort);
  gather    out[i] = weights[g_i], compared in full;
  backward  integer-valued gradients, so every summation order gives the same exact fp32 sums: the
            rows and their sums must equal an int64 index_add of the same lookups.
"""
import os
import time

import numpy as np
import pytest
import torch

from helpers import entry

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

N_MAX = (1 << 31) - 1

def _progress(msg):
    """Progress line for long tests: stdout (visible with -s) and, if FS_TEST_PROGRESS_FILE names a file,
    a line appended there, so that a quiet minute of a long test is not mistaken for a hang."""
    print(msg, flush=True)
    path = os.environ.get("FS_TEST_PROGRESS_FILE")
    if path:
        try:
            with open(path, "a") as f:
                f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
        except OSError:
            pass


def test_two_billion_lookups():
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < 200e9:
        pytest.skip(f"needs ~200 GB of free HBM, {free_b / 1e9:.0f} GB free")
    n, R, D, U, W, self_ = N_MAX, 1 << 20, 4, 16, 4, 5
    T, B = 2, 1 << 15
    E = R // T
    gen = torch.Generator(device=dev).manual_seed(7)
    _progress(f"[max] generating {n} lookups")
    # segment lengths: equal, the remainder on the last one; ids uniform inside each table
    S = T * B
    lengths = torch.full((S,), n // S, dtype=torch.int64, device=dev)
    lengths[-1] += n - int(lengths.sum())
    offsets = torch.zeros(S + 1, dtype=torch.int64, device=dev)
    offsets[1:] = torch.cumsum(lengths, 0)
    assert int(offsets[-1]) == n
    ids = torch.randint(0, E, (n,), dtype=torch.int64, device=dev, generator=gen)
    row_base = torch.tensor([0, E, 2 * E], dtype=torch.int64, device=dev)
    tier = torch.randint(0, 3, (R,), dtype=torch.int64, device=dev, generator=gen)
    owner = torch.where(tier == 2, torch.randint(0, U, (R,), device=dev, generator=gen),
                        torch.randint(0, W, (R,), device=dev, generator=gen))
    placement = ((tier << 30) | owner).to(torch.int32)          # bit 31 set for tier 2: same 32 bits
    dest_of_row = torch.where(tier == 0, self_, torch.where(tier == 1, (self_ // W) * W + owner, owner)).to(torch.int16)
    first_of_table1 = int(offsets[B])                            # lookups before it belong to table 0

    # ---------------------------------------------------------------- route
    _progress("[max] route")
    bo = torch.zeros(U + 1, dtype=torch.int64, device=dev)
    rows = torch.empty(n, dtype=torch.int64, device=dev)
    pos = torch.empty(n, dtype=torch.int32, device=dev)
    tc = torch.zeros(3, dtype=torch.int64, device=dev)
    st = torch.zeros(1, dtype=torch.int32, device=dev)
    assert fs.fs_route_bucketize(ids, offsets, T, B, row_base, placement, n, U, W, self_, bo, rows, pos, tc, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    _progress("[max] route: properties")
    step = 1 << 27
    counts = torch.zeros(U, dtype=torch.int64, device=dev)
    tiers = torch.zeros(3, dtype=torch.int64, device=dev)
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        g = ids[lo:hi] + torch.where(torch.arange(lo, hi, device=dev) >= first_of_table1, E, 0)
        counts += torch.bincount(dest_of_row[g].long(), minlength=U)
        tiers += torch.bincount(tier[g], minlength=3)
    assert torch.equal(bo[1:] - bo[:-1], counts) and int(bo[0]) == 0 and int(bo[-1]) == n
    assert torch.equal(tc, tiers)
    bo_h = bo.cpu().tolist()
    bucket_start = torch.zeros(n + 1, dtype=torch.bool, device=dev)
    bucket_start[torch.as_tensor(bo_h, device=dev)] = True
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        p = pos[lo:hi].long()
        g = ids[p] + torch.where(p >= first_of_table1, E, 0)
        assert torch.equal(rows[lo:hi], g), lo                                    # the pair is a lookup of the batch
        b_of_j = torch.bucketize(torch.arange(lo, hi, device=dev), bo[1:], right=True)
        assert torch.equal(dest_of_row[g].long(), b_of_j), lo                      # in the bucket of its destination
        if hi - lo > 1:
            asc = p[1:] > p[:-1]
            assert torch.all(asc | bucket_start[lo + 1:hi]), lo                    # ascending inside a bucket
        if lo > 0:
            assert int(pos[lo]) > int(pos[lo - 1]) or bool(bucket_start[lo])
    del bucket_start, counts
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- the shared sort
    _progress("[max] sort of the lookups")
    srows = torch.empty(n, dtype=torch.int32, device=dev)
    spos = torch.empty(n, dtype=torch.int32, device=dev)
    assert fs.fs_sort_lookups(rows, pos, 0, n, R, n, srows, spos, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    _progress("[max] sort: properties")
    per_row = torch.zeros(R, dtype=torch.int64, device=dev)
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        r, p = srows[lo:hi].long(), spos[lo:hi].long()
        g = ids[p] + torch.where(p >= first_of_table1, E, 0)
        assert torch.equal(r, g), lo                                              # every pair is a lookup of the batch
        per_row += torch.bincount(r, minlength=R)
        if hi - lo > 1:
            up = (r[1:] > r[:-1]) | ((r[1:] == r[:-1]) & (p[1:] > p[:-1]))         # (row, pos) strictly ascending,
            assert bool(up.all()), lo                                             # so no lookup appears twice
        if lo > 0:
            r0, p0 = int(srows[lo - 1]), int(spos[lo - 1])
            assert (int(srows[lo]), int(spos[lo])) > (r0, p0)
    for lo in range(0, n, step):                                                  # ... and every lookup once: the rows' counts
        hi = min(n, lo + step)
        per_row -= torch.bincount(rows[lo:hi], minlength=R)
    assert not bool(per_row.any())
    del per_row
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- gather (16-byte rows)
    _progress("[max] gather")
    weights = torch.randn(R, D, device=dev, generator=gen)
    out = torch.empty(n, D, dtype=torch.float32, device=dev)
    assert fs.fs_seq_gather_fwd(weights, rows, pos, 0, n, out, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    _progress("[max] gather: full compare")
    w_bits, out_bits = weights.view(torch.int32), out.view(torch.int32)
    small = 1 << 24                      # torch's row gather refuses 2^27 indices in one call
    for lo in range(0, n, small):
        hi = min(n, lo + small)
        g = ids[lo:hi] + torch.where(torch.arange(lo, hi, device=dev) >= first_of_table1, E, 0)
        ref = torch.index_select(w_bits, 0, g)
        assert not bool((out_bits[lo:hi] != ref).any()), lo
    del ref
    # the gather in row order over the same lookups: the same bits (checked a half of the output at a time
    # against the copy the first gather wrote, so that no second output buffer is needed)
    _progress("[max] gather in row order")
    half = n // 2
    for lo_h, hi_h in ((0, half), (half, n)):
        keep = out_bits[lo_h:hi_h].clone()
        out[lo_h:hi_h].zero_()
        inside = (spos >= lo_h) & (spos < hi_h)
        sr_h, sp_h = srows[inside].contiguous(), spos[inside].contiguous()
        del inside
        assert sr_h.numel() == hi_h - lo_h
        assert fs.fs_seq_gather_fwd_sorted(weights, sr_h, sp_h, sr_h.numel(), out, st) == 0
        torch.cuda.synchronize()
        assert int(st.item()) == 0 and torch.equal(out_bits[lo_h:hi_h], keep), lo_h
        del keep, sr_h, sp_h
    del out, weights, ids, w_bits, out_bits
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- backward, integer-valued gradients
    _progress("[max] backward")
    grad = torch.randint(-2, 3, (n, D), device=dev, generator=gen, dtype=torch.int8).float()
    uniq = torch.empty(R, dtype=torch.int64, device=dev)
    rg = torch.empty(R, D, dtype=torch.float32, device=dev)
    nu = torch.zeros(1, dtype=torch.int64, device=dev)
    assert fs.fs_seq_grad_bwd(grad, rows, pos, 0, n, R, 0, uniq, rg, R, nu, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    _progress("[max] backward: exact sums")
    want = torch.zeros(R, D, dtype=torch.int64, device=dev)
    seen = torch.zeros(R, dtype=torch.int64, device=dev)
    for lo in range(0, n, small):
        hi = min(n, lo + small)
        r = rows[lo:hi]
        want.index_add_(0, r, torch.index_select(grad, 0, pos[lo:hi].long()).long())
        seen += torch.bincount(r, minlength=R)
    present = torch.nonzero(seen > 0).flatten()
    k = int(nu.item())
    assert k == present.numel() and torch.equal(uniq[:k], present)
    assert int(want.abs().max()) < (1 << 24)                                       # every sum is an exact fp32 integer
    assert torch.equal(rg[:k].long(), want[present]) and torch.equal(rg[:k], rg[:k].round())
    # the backward on the shared sort's pairs: the same rows, the same bits
    _progress("[max] backward on the sorted pairs")
    del want, seen
    uniq_s = torch.empty(R, dtype=torch.int64, device=dev)
    rg_s = torch.empty(R, D, dtype=torch.float32, device=dev)
    assert fs.fs_seq_grad_bwd_sorted(grad, srows, spos, n, R, 0, uniq_s, rg_s, R, nu, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0 and int(nu.item()) == k
    assert torch.equal(uniq_s[:k], uniq[:k]) and torch.equal(rg_s[:k].view(torch.int32), rg[:k].view(torch.int32))
    _progress("[max] done")


def test_largest_table_row_ids():
    """R = 2^32 - 2 rows, the largest table the interface admits: placement and counts are 17 GB each, the lookups
    aim at both ends of each table and at the rows either side of 2^31.  The oracle runs on the same ids with a
    placement given as the few entries that differ from the constant background (it never reads the others)."""
    import oracle
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < 120e9:
        pytest.skip(f"needs ~120 GB of free HBM, {free_b / 1e9:.0f} GB free")
    R = (1 << 32) - 2
    T, B, U, W, self_ = 2, 64, 8, 4, 6
    E = R // T                                                     # 2^31 - 1 rows per table
    rng = np.random.default_rng(11)
    S = T * B
    lengths = rng.integers(0, 200, S)
    offsets = np.zeros(S + 1, np.int64)
    np.cumsum(lengths, out=offsets[1:])
    n = int(offsets[-1])
    special = np.array([0, 1, E - 1, E - 2, E // 2, (1 << 30), (1 << 30) - 1, 12345, E - 12345], np.int64)
    ids = np.where(rng.random(n) < 0.6, special[rng.integers(0, len(special), n)], rng.integers(0, E, n)).astype(np.int64)
    row_base = np.array([0, E, 2 * E], np.int64)
    table = np.searchsorted(offsets[::B][1:], np.arange(n), side="right")
    g = row_base[table] + ids                                      # global rows: up to 2^32 - 3
    assert g.max() == R - 1 and g.min() == 0 and (g >= (1 << 31)).any() and (g < (1 << 31)).any()
    # placement: tier 2 / owner 3 everywhere, except the rows this batch touches (random tiers and owners)
    _progress("[max R] placement and counts, 17 GB each")
    pl_d = torch.full((R,), entry(2, 3) - (1 << 32), dtype=torch.int32, device=dev)
    touched = np.unique(g)
    tiers = rng.integers(0, 3, len(touched))
    owners = np.where(tiers == 2, rng.integers(0, U, len(touched)), rng.integers(0, W, len(touched)))
    vals = ((tiers.astype(np.int64) << 30) | owners).astype(np.uint32)
    pl_d[torch.from_numpy(touched).to(dev)] = torch.from_numpy(vals.view(np.int32)).to(dev)
    # the oracle's placement: a compact table over the touched rows, the batch re-indexed into it
    local = np.searchsorted(touched, g)
    o_rc, o_st, o_bo, o_rows, o_pos, o_tc = oracle.route_bucketize(local, np.array([0, n], np.int64), 1, 1,
                                                                   np.array([0, len(touched)], np.int64), vals, U, W, self_, n=n)
    assert (o_rc, o_st) == (0, 0)
    bo = torch.zeros(U + 1, dtype=torch.int64, device=dev)
    rows = torch.empty(n, dtype=torch.int64, device=dev)
    pos = torch.empty(n, dtype=torch.int32, device=dev)
    tc = torch.zeros(3, dtype=torch.int64, device=dev)
    st = torch.zeros(1, dtype=torch.int32, device=dev)
    ids_d, off_d, rb_d = (torch.from_numpy(a).to(dev) for a in (ids, offsets, row_base))
    _progress("[max R] route")
    assert fs.fs_route_bucketize(ids_d, off_d, T, B, rb_d, pl_d, n, U, W, self_, bo, rows, pos, tc, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    assert np.array_equal(bo.cpu().numpy(), o_bo) and np.array_equal(tc.cpu().numpy(), o_tc)
    assert np.array_equal(pos.cpu().numpy(), o_pos)
    assert np.array_equal(rows.cpu().numpy(), touched[o_rows])                     # the oracle's rows are indices into touched
    del pl_d
    torch.cuda.empty_cache()
    # histogram over the same ids: counts[g] += 1, everything else stays 0
    _progress("[max R] histogram")
    counts = torch.zeros(R, dtype=torch.int32, device=dev)
    assert fs.fs_plan_replication(ids_d, off_d, T, B, rb_d, n, R, counts, fs.FS_PLAN_ACCUMULATE, dev_status=st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    want = np.bincount(local, minlength=len(touched))
    assert np.array_equal(counts[torch.from_numpy(touched).to(dev)].cpu().numpy(), want)
    assert int(counts.sum(dtype=torch.int64).item()) == n
    # top-k under a budget and the tier cuts on those counts (workspaces of ~90 GB: four 17 GB sort buffers and
    # the per-tile tables); the oracle sees the touched rows only, whose order is the global one
    free_b, _ = torch.cuda.mem_get_info()
    if free_b > 130e9:
        _progress("[max R] select and tiers")
        k_budget = len(touched) // 2
        sel = torch.full((k_budget,), -1, dtype=torch.int64, device=dev)
        nsel = torch.zeros(1, dtype=torch.int64, device=dev)
        assert fs.fs_plan_replication(None, None, 1, 1, None, 0, R, counts, fs.FS_PLAN_SELECT, k_budget * 16, 16, sel, nsel,
                                      dev_status=st) == 0
        torch.cuda.synchronize()
        o_rc, o_st, o_sel = oracle.plan_replication(None, None, 1, 1, None, len(touched), want.astype(np.uint32),
                                                    oracle.PLAN_SELECT, k_budget * 16, 16)
        assert o_rc == 0 and int(nsel.item()) == len(o_sel) == k_budget
        assert np.array_equal(sel.cpu().numpy(), touched[o_sel])
        del sel
        torch.cuda.empty_cache()
        tp = dict(num_samples=B, B=4, U=U, W=W, dp_multiplier=6, granule=1, a2a_global=1, a2a_intra=6, ar_global=3, ar_cross=2)
        cuts = torch.zeros(fs.FS_TIER_CUTS, dtype=torch.int64, device=dev)
        srt = torch.full((len(touched),), -1, dtype=torch.int64, device=dev)
        assert fs.fs_plan_tiers(counts, R, tp, 3, srt, len(touched), cuts) == 0
        torch.cuda.synchronize()
        o_rc, o_cuts, o_rows = oracle.plan_tiers(want.astype(np.uint32), tp, 3, cap=len(touched))
        assert o_rc == 0 and cuts.cpu().numpy().tolist() == o_cuts.tolist()
        assert np.array_equal(srt.cpu().numpy()[:len(o_rows)], touched[o_rows])
        del srt
    del counts
    torch.cuda.empty_cache()
    # backward on the routed lists: row ids that need all 32 key bits
    _progress("[max R] backward")
    D = 4
    grad = torch.from_numpy(rng.integers(-3, 4, (n, D)).astype(np.float32)).to(dev)
    uniq = torch.empty(len(touched), dtype=torch.int64, device=dev)
    rg = torch.empty(len(touched), D, dtype=torch.float32, device=dev)
    nu = torch.zeros(1, dtype=torch.int64, device=dev)
    assert fs.fs_seq_grad_bwd(grad, rows, pos, 0, n, R, 0, uniq, rg, len(touched), nu, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == 0 and int(nu.item()) == len(touched)
    assert np.array_equal(uniq.cpu().numpy(), touched)
    sums = np.zeros((len(touched), D))
    np.add.at(sums, local, grad.cpu().numpy().astype(np.float64))
    assert np.array_equal(rg.cpu().numpy().astype(np.float64), sums)              # small integers: exact in fp32
    _progress("[max R] done")
