"""Randomised end-to-end parity: random shapes, dtypes, bucket counts, length laws with empty segments,
per-bucket and arbitrary [j0, j1) ranges, both backward variants, capacities below the number of distinct
rows -- route + bucketize, gather and backward against the CPU oracle on exactly the same inputs."""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle
from helpers import random_placement

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def _case(rng):
    dt = str(rng.choice(["f32", "f16", "bf16"]))
    unit = 4 if dt == "f32" else 8
    D = int(unit * rng.choice([1, 2, 3, 8, 16, 32, 33, 64, 130]))
    U = int(rng.choice([1, 2, 8, 24, 64, 256]))
    W = int(rng.choice([w for w in (1, 2, 4, 8, 64) if U % w == 0]))
    T = int(rng.integers(1, 5))
    B = int(rng.integers(1, 300))
    E = int(rng.choice([7, 300, 5000, 70000]))
    law = rng.choice(["fixed", "uniform", "heavy", "mostly-empty"])
    S = T * B
    if law == "fixed":
        lengths = np.full(S, int(rng.integers(0, 40)))
    elif law == "uniform":
        lengths = rng.integers(0, 120, S)
    elif law == "heavy":
        lengths = np.minimum(rng.pareto(0.8, S) * 8, 3000).astype(np.int64)
    else:
        lengths = np.where(rng.random(S) < 0.9, 0, rng.integers(1, 500, S))
    offsets = np.zeros(S + 1, np.int64)
    np.cumsum(lengths, out=offsets[1:])
    n = int(offsets[-1])
    skew = rng.choice([0.0, 1.0, 1.6])
    if skew == 0.0:
        ids = rng.integers(0, E, n)
    else:
        ids = np.minimum((rng.pareto(skew, n)).astype(np.int64), E - 1)
        ids = rng.permutation(E)[ids]
    return dict(dt=dt, D=D, U=U, W=W, T=T, B=B, E=E, n=n, self_=int(rng.integers(0, U)), offsets=offsets,
                ids=ids.astype(np.int64), row_base=(np.arange(T + 1) * E).astype(np.int64),
                placement=random_placement(rng, T * E, U, W, p=rng.dirichlet([1, 1, 1])))


@pytest.mark.parametrize("seed", range(60))
def test_random_pipeline(G, seed):
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(1000 + seed)
    c = _case(rng)
    n, R, D, dt = c["n"], c["T"] * c["E"], c["D"], c["dt"]
    code = G.oracle_dtype(dt)
    # ---- route
    rc, st, bo, rows, pos, tc = G.hip_route(G.to_dev(c["ids"], torch.int64), G.to_dev(c["offsets"], torch.int64), c["T"],
                                            c["B"], G.to_dev(c["row_base"], torch.int64), G.placement_dev(c["placement"]),
                                            c["U"], c["W"], c["self_"], n=n)
    orc, ost, obo, orows, opos, otc = oracle.route_bucketize(c["ids"], c["offsets"], c["T"], c["B"], c["row_base"],
                                                             c["placement"], c["U"], c["W"], c["self_"], n=n)
    assert (rc, st) == (orc, ost) == (0, 0)
    assert np.array_equal(bo.cpu().numpy(), obo) and np.array_equal(tc.cpu().numpy(), otc)
    assert np.array_equal(rows.cpu().numpy(), orows) and np.array_equal(pos.cpu().numpy(), opos)
    # ---- the router that also hands over the slot a replicated row's placement entry carries
    bo_s = torch.zeros(c["U"] + 1, dtype=torch.int64, device=G.DEV)
    rows_s = torch.zeros(max(n, 1), dtype=torch.int64, device=G.DEV)
    pos_s = torch.zeros(max(n, 1), dtype=torch.int32, device=G.DEV)
    slots_s = torch.full((max(n, 1),), -7, dtype=torch.int32, device=G.DEV)
    tc_s = torch.zeros(3, dtype=torch.int64, device=G.DEV)
    st_s = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    assert fs.fs_route_bucketize_slots(G.to_dev(c["ids"], torch.int64), G.to_dev(c["offsets"], torch.int64), c["T"], c["B"],
                                       G.to_dev(c["row_base"], torch.int64), G.placement_dev(c["placement"]), n, c["U"], c["W"],
                                       c["self_"], bo_s, rows_s, pos_s, slots_s, tc_s, st_s) == 0
    orc, ost, oslots = oracle.lookup_slots(c["placement"], orows, 0, n)
    torch.cuda.synchronize()
    assert (orc, ost) == (0, 0) and int(st_s.item()) == 0
    assert np.array_equal(bo_s.cpu().numpy(), obo) and np.array_equal(tc_s.cpu().numpy(), otc)
    assert np.array_equal(rows_s[:n].cpu().numpy(), orows) and np.array_equal(pos_s[:n].cpu().numpy(), opos)
    assert np.array_equal(slots_s[:n].cpu().numpy(), oslots)
    if n == 0:
        return
    # ---- ranges: everything, one bucket, an arbitrary slice, an empty range
    b = int(rng.integers(0, c["U"]))
    a1, a2 = sorted(int(x) for x in rng.integers(0, n + 1, 2))
    ranges = [(0, n), (int(obo[b]), int(obo[b + 1])), (a1, a2), (a1, a1)]
    Wt = (torch.randn(R, D, generator=torch.Generator().manual_seed(seed)) * 3).to(TDT[dt])
    Wn = fs_inputs.as_numpy_bits(Wt)
    W_d = Wt.to(G.DEV)
    grad = torch.randn(n, D, generator=torch.Generator().manual_seed(seed + 1)).to(TDT[dt])
    grad_n = fs_inputs.as_numpy_bits(grad)
    grad_d = grad.to(G.DEV)
    st_d = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    for j0, j1 in ranges:
        # gather
        out = torch.full((n, D), 5.0, dtype=TDT[dt], device=G.DEV)
        assert fs.fs_seq_gather_fwd(W_d, rows, pos, j0, j1, out, st_d) == 0
        ref = fs_inputs.as_numpy_bits(torch.full((n, D), 5.0, dtype=TDT[dt])).copy()
        assert oracle.seq_gather_fwd(Wn, orows, opos, j0, j1, ref, dtype=code) == (0, 0)
        torch.cuda.synchronize()
        assert np.array_equal(G.bits(out), ref.view(np.uint8).reshape(-1)), (j0, j1)
        # backward, sorted variant: bit for bit; a capacity below the number of distinct rows cuts the lists
        orc, ost, ou, og, og64, onu = oracle.seq_grad_bwd(grad_n, orows, opos, j0, j1, R, dtype=code)
        rc, st, u, g, nu = G.hip_bwd(grad_d, rows, pos, j0, j1, R, 0)
        assert (rc, st, nu) == (orc, ost, onu)
        assert np.array_equal(u.cpu().numpy(), ou)
        assert np.array_equal(g.cpu().numpy().view(np.uint32), og.view(np.uint32)), (j0, j1)
        # the shared sort and the entry points that take its pairs: the oracle's order, then the same bits
        m = j1 - j0
        srows = torch.zeros(max(m, 1), dtype=torch.int32, device=G.DEV)
        spos = torch.zeros(max(m, 1), dtype=torch.int32, device=G.DEV)
        assert fs.fs_sort_lookups(rows, pos, j0, j1, R, n, srows, spos, st_d) == 0
        orc, ost, osr, osp = oracle.sort_lookups(orows, opos, j0, j1, R, n)
        assert (orc, ost) == (0, 0)
        assert np.array_equal(srows[:m].cpu().numpy().view(np.uint32), osr)
        assert np.array_equal(spos[:m].cpu().numpy().view(np.uint32), osp)
        us = torch.full((max(onu, 1),), -7, dtype=torch.int64, device=G.DEV)
        gs = torch.full((max(onu, 1), D), float("nan"), dtype=torch.float32, device=G.DEV)
        nus = torch.full((1,), -7, dtype=torch.int64, device=G.DEV)
        assert fs.fs_seq_grad_bwd_sorted(grad_d, srows, spos, m, R, 0, us, gs, max(onu, 1), nus, st_d) == 0
        assert int(nus.item()) == onu and np.array_equal(us[:onu].cpu().numpy(), ou)
        assert np.array_equal(gs[:onu].cpu().numpy().view(np.uint32), og.view(np.uint32)), (j0, j1)
        out_s = torch.full((n, D), 5.0, dtype=TDT[dt], device=G.DEV)
        assert fs.fs_seq_gather_fwd_sorted(W_d, srows, spos, m, out_s, st_d) == 0
        torch.cuda.synchronize()
        assert np.array_equal(G.bits(out_s), ref.view(np.uint8).reshape(-1)), (j0, j1)
        if onu > 1:
            cap = int(rng.integers(1, onu))
            rc, st, u, g, nu = G.hip_bwd(grad_d, rows, pos, j0, j1, R, 0, cap)
            assert rc == 0 and st == oracle.UNIQUE_OVERFLOW and nu == onu
            assert np.array_equal(u.cpu().numpy(), ou[:cap])
            assert np.array_equal(g.cpu().numpy().view(np.uint32), og[:cap].view(np.uint32))
        # atomic variant: within 1e-5 of the fp64 sums, relative to max(|sum|, 2-norm of the terms)
        rc, st, u1, g1, nu1 = G.hip_bwd(grad_d, rows, pos, j0, j1, R, 1)
        assert (rc, st, nu1) == (0, 0, onu) and np.array_equal(u1.cpu().numpy(), ou)
        if onu:
            sq = np.zeros((onu, D))
            terms = grad_n[opos[j0:j1]]
            terms = (terms.astype(np.uint32) << 16).view(np.float32) if dt == "bf16" else terms
            np.add.at(sq, np.searchsorted(ou, orows[j0:j1]), terms.astype(np.float64) ** 2)
            assert np.all(np.abs(g1.cpu().numpy() - og64) <= 1e-5 * np.maximum(np.abs(og64), np.sqrt(sq)))
    assert int(st_d.item()) == 0
