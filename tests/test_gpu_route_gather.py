"""GPU parity: fs_route_bucketize and fs_seq_gather_fwd against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle
from helpers import entry, random_jagged, random_placement

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def _route_both(G, ids, offsets, T, B, row_base, placement, U, W, self_, n=None):
    rc, st, bo, rows, pos, tc = G.hip_route(G.to_dev(ids, torch.int64), G.to_dev(offsets, torch.int64), T, B,
                                            G.to_dev(row_base, torch.int64), G.placement_dev(placement), U, W, self_, n=n)
    orc, ost, obo, orows, opos, otc = oracle.route_bucketize(ids, offsets, T, B, row_base, placement, U, W, self_, n=n)
    return (rc, st, bo.cpu().numpy(), rows.cpu().numpy(), pos.cpu().numpy(), tc.cpu().numpy()), (orc, ost, obo, orows, opos, otc)


def _assert_same_route(h, o):
    assert h[0] == o[0] and h[1] == o[1]
    for a, b in zip(h[2:], o[2:]):
        assert np.array_equal(a, b)


def test_route_c1(G):
    cfg = fs_inputs.CONFIGS["c1"]
    b, pl = G.batch_on(cfg, "cpu")
    h, o = _route_both(G, b["ids"].numpy(), b["offsets"].numpy(), cfg.T, cfg.B, b["row_base"].numpy(),
                       pl.numpy().view(np.uint32), cfg.U, cfg.W, cfg.self_bucket)
    _assert_same_route(h, o)
    assert h[2][-1] == 8192


@pytest.mark.parametrize("case", [
    dict(T=3, B=37, E=500, L=60, U=8, W=4, s=5),         # ~3 tiles, ragged tail
    dict(T=1, B=300, E=4000, L=90, U=64, W=8, s=17),     # several tiles, 64 buckets
    dict(T=16, B=9, E=100, L=200, U=128, W=128, s=0),    # tiles that span many tables
    dict(T=2, B=50, E=300, L=130, U=1, W=1, s=0),        # one bucket
    dict(T=2, B=64, E=9000, L=100, U=4096, W=64, s=4095),  # maximum bucket count
    dict(T=5, B=3, E=50, L=3, U=6, W=3, s=2),            # smaller than one wave's span
])
def test_route_random(G, case):
    rng = np.random.default_rng(case["U"] * 1000 + case["T"])
    ids, offsets, row_base, n = random_jagged(rng, case["T"], case["B"], case["E"], case["L"])
    pl = random_placement(rng, case["T"] * case["E"], case["U"], case["W"])
    h, o = _route_both(G, ids, offsets, case["T"], case["B"], row_base, pl, case["U"], case["W"], case["s"])
    _assert_same_route(h, o)


def test_route_skewed_three_tier(G):
    """c3's laws on a table the oracle sorts in seconds: ~90 % of lookups land in one bucket."""
    cfg = fs_inputs.CONFIGS["c3"].scaled(E=200_000, B=256, T=4)
    b, pl = G.batch_on(cfg, "cpu")
    h, o = _route_both(G, b["ids"].numpy(), b["offsets"].numpy(), cfg.T, cfg.B, b["row_base"].numpy(),
                       pl.numpy().view(np.uint32), cfg.U, cfg.W, 13)
    _assert_same_route(h, o)
    assert h[5][1] > 0            # tier 1 is exercised


def test_route_edges_and_faults(G):
    # empty batch
    h, o = _route_both(G, np.zeros(0, np.int64), np.zeros(7, np.int64), 2, 3, np.array([0, 4, 8]), np.zeros(8, np.uint32), 5, 1, 2)
    assert h[0] == 0 and h[1] == 0 and np.array_equal(h[2], o[2]) and np.array_equal(h[5], o[5])
    # data faults: bad ids, bad owners, tier 3
    rng = np.random.default_rng(4)
    ids, offsets, row_base, n = random_jagged(rng, 2, 40, 100, 90)
    ids[rng.integers(0, n, 50)] = 100 + rng.integers(0, 5, 50)
    ids[rng.integers(0, n, 20)] = -3
    pl = random_placement(rng, 200, 8, 4)
    pl[::7] = entry(3, 1)
    pl[1::11] = entry(2, 8)
    pl[2::13] = entry(1, 4)
    h, o = _route_both(G, ids, offsets, 2, 40, row_base, pl, 8, 4, 6)
    _assert_same_route(h, o)
    assert h[1] == (oracle.BAD_ID | oracle.BAD_PLACEMENT)
    # bad offsets: flagged, outputs unspecified, nothing out of bounds (the call returns)
    bad = offsets.copy()
    bad[5] = bad[6] + 3
    h, o = _route_both(G, ids, bad, 2, 40, row_base, pl, 8, 4, 6, n=n)
    assert h[0] == 0 and h[1] & oracle.BAD_OFFSETS and o[1] & oracle.BAD_OFFSETS
    h, o = _route_both(G, ids, offsets, 2, 40, row_base, pl, 8, 4, 6, n=n - 1)
    assert h[1] & oracle.BAD_OFFSETS and o[1] & oracle.BAD_OFFSETS


def test_route_host_faults(G):
    import paper_2301_02959_amd as fs
    ids, offsets, rb = G.to_dev([0], torch.int64), G.to_dev([0, 1], torch.int64), G.to_dev([0, 2], torch.int64)
    pl = G.placement_dev(np.zeros(2, np.uint32))
    bo = torch.zeros(5, dtype=torch.int64, device=G.DEV)
    r = torch.zeros(1, dtype=torch.int64, device=G.DEV)
    p = torch.zeros(1, dtype=torch.int32, device=G.DEV)

    def call(T=1, B=1, n=1, U=2, W=1, s=0, ws=None, offs=offsets):
        return fs.fs_route_bucketize(ids, offs, T, B, rb, pl, n, U, W, s, bo, r, p, None, None, workspace=ws,
                                     raise_on_error=False)
    assert call() == 0
    assert call(n=-1) == 2 and call(T=0) == 2 and call(B=0) == 2 and call(n=1 << 31) == 2
    assert call(U=0) == 6 and call(U=4097) == 6 and call(W=0) == 6 and call(U=4, W=3) == 6 and call(s=2) == 6
    assert call(ws=torch.zeros(256, dtype=torch.uint8, device=G.DEV)[:16]) == 5      # too small
    assert call(offs=None, ws=torch.zeros(1 << 16, dtype=torch.uint8, device=G.DEV)) == 1
    with pytest.raises(fs.FlexShardError):
        fs.fs_route_bucketize(ids, offsets, 1, 1, rb, pl, 1, 0, 1, 0, bo, r, p)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ gather
@pytest.mark.parametrize("dt,D", [("f32", 4), ("f32", 64), ("f16", 8), ("f16", 128), ("bf16", 256), ("f16", 24),
                                  ("bf16", 512), ("f32", 520), ("f16", 1024 + 64)])
def test_gather_bit_exact(G, dt, D):
    rng = np.random.default_rng(D)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dt]
    R, n = 3000, 5003                                   # several tiles at every row size + ragged tail
    Wt = torch.randn(R, D, generator=torch.Generator().manual_seed(D)).to(tdt)
    g = rng.integers(0, R, n)
    perm = rng.permutation(n).astype(np.int32)
    rows = g[perm]
    out = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    import paper_2301_02959_amd as fs
    rows_d, pos_d, W_d = G.to_dev(rows, torch.int64), G.to_dev(perm, torch.int32), Wt.to(G.DEV)
    assert fs.fs_seq_gather_fwd(W_d, rows_d, pos_d, 0, n, out, st) == 0
    torch.cuda.synchronize()
    Wn = fs_inputs.as_numpy_bits(Wt)
    ref = np.zeros_like(Wn, shape=(n, D))
    assert oracle.seq_gather_fwd(Wn, rows, perm, 0, n, ref, dtype=G.oracle_dtype(dt)) == (0, 0)
    assert int(st.item()) == 0 and np.array_equal(G.bits(out), ref.view(np.uint8).reshape(-1))
    # the textbook lookup
    assert torch.equal(out, W_d[torch.as_tensor(g, device=G.DEV)])
    # partial range: untouched rows keep the sentinel
    out2 = torch.full((n, D), 7.0, dtype=tdt, device=G.DEV)
    assert fs.fs_seq_gather_fwd(W_d, rows_d, pos_d, 1234, 4321, out2, st) == 0
    ref2 = fs_inputs.as_numpy_bits(torch.full((n, D), 7.0, dtype=tdt)).copy()
    oracle.seq_gather_fwd(Wn, rows, perm, 1234, 4321, ref2, dtype=G.oracle_dtype(dt))
    assert np.array_equal(G.bits(out2), ref2.view(np.uint8).reshape(-1))


def test_gather_faults(G):
    import paper_2301_02959_amd as fs
    Wt = torch.arange(8 * 4, dtype=torch.float32).reshape(8, 4).to(G.DEV)
    out = torch.full((3, 4), -1.0, device=G.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    rows, pos = G.to_dev([1, 9, 2, -1, 3], torch.int64), G.to_dev([0, 1, 5, 2, 2], torch.int32)
    assert fs.fs_seq_gather_fwd(Wt, rows, pos, 0, 5, out, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID
    assert torch.equal(out[0], Wt[1]) and torch.all(out[1] == -1) and torch.equal(out[2], Wt[3])
    assert fs.fs_seq_gather_fwd(Wt, rows, pos, 2, 2, out, st) == 0                       # empty range
    assert fs.fs_seq_gather_fwd(Wt, rows, pos, 3, 2, out, st, raise_on_error=False) == 2
    assert fs.fs_seq_gather_fwd(Wt, rows, pos, 0, 1, out, st, raise_on_error=False, D=3) == 4
    assert fs.fs_seq_gather_fwd(Wt, rows, pos, 0, 1, out, st, raise_on_error=False, dtype=9) == 3
    assert fs.fs_seq_gather_fwd(Wt, None, pos, 0, 1, out, st, raise_on_error=False) == 1
    misaligned = torch.zeros(3 * 4 + 1, device=G.DEV)[1:].view(3, 4)
    assert fs.fs_seq_gather_fwd(Wt, rows, pos, 0, 1, misaligned, st, raise_on_error=False) == 4


def test_route_then_gather_c1_end_to_end(G):
    import paper_2301_02959_amd as fs
    cfg = fs_inputs.CONFIGS["c1"]
    b, pl = G.batch_on(cfg, "cpu")
    Wt = fs_inputs.make_table(cfg)
    rc, st, bo, rows, pos, tc = G.hip_route(b["ids"].to(G.DEV), b["offsets"].to(G.DEV), cfg.T, cfg.B,
                                            b["row_base"].to(G.DEV), pl.to(G.DEV), cfg.U, cfg.W, 0)
    out = torch.zeros(b["n"], cfg.D, device=G.DEV)
    fs.fs_seq_gather_fwd(Wt.to(G.DEV), rows, pos, 0, b["n"], out)
    torch.cuda.synchronize()
    assert torch.equal(out.cpu(), Wt[b["ids"]])           # T = 1: global row = id
    # only this GPU's bucket: the other lookups stay untouched
    out = torch.full((b["n"], cfg.D), 5.0, device=G.DEV)
    lo, hi = int(bo[0]), int(bo[1])
    fs.fs_seq_gather_fwd(Wt.to(G.DEV), rows, pos, lo, hi, out)
    mine = torch.zeros(b["n"], dtype=torch.bool)
    mine[pos[lo:hi].cpu().long()] = True
    assert torch.equal(out.cpu()[mine], Wt[b["ids"]][mine]) and torch.all(out.cpu()[~mine] == 5.0)


def test_route_row_base_out_of_order_stays_in_bounds(G):
    """A row_base that is not ascending takes lookups out of [0, row_base[T]): they are routed as row 0
    and reported, every output stays in range."""
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(77)
    T, B, U, W = 2, 40, 8, 4
    ids, offsets, _, n = random_jagged(rng, T, B, 50, 30)
    row_base = np.array([0, 100, 50], dtype=np.int64)            # table 1 would start past the end
    pl = random_placement(rng, 50, U, W)                          # row_base[T] = 50 placement entries
    rc, st, bo, rows, pos, tc = G.hip_route(G.to_dev(ids, torch.int64), G.to_dev(offsets, torch.int64), T, B,
                                            G.to_dev(row_base, torch.int64), G.placement_dev(pl), U, W, 3, n=n)
    assert rc == 0 and st & fs.FS_DEV_BAD_ID
    rows = rows.cpu().numpy(); pos = pos.cpu().numpy(); bo = bo.cpu().numpy()
    assert rows.min() >= 0 and rows.max() < 50
    assert np.array_equal(np.sort(pos), np.arange(n))
    assert bo[0] == 0 and bo[-1] == n and np.all(np.diff(bo) >= 0)
    second = np.arange(n) >= offsets[B]                           # lookups of table 1
    assert np.all(rows[np.isin(pos, np.nonzero(second)[0])] == 0)
