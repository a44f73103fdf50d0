"""GPU parity: fs_plan_tiers against the CPU oracle, exact (every cut, the chosen rows in order,
the tags)."""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle
from helpers import entry

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def params(**kw):
    p = dict(num_samples=1000, B=16, U=8, W=4, dp_multiplier=6, granule=1,
             a2a_global=10, a2a_intra=40, ar_global=30, ar_cross=20)
    p.update(kw)
    return p


def both(G, counts, p, tiers, cap=None, tag=True):
    import paper_2301_02959_amd as fs
    R = len(counts)
    cap = R if cap is None else cap
    pl0 = np.full(R, entry(2, 1), np.uint32)
    pl0[::3] = entry(0, 7)
    o_pl = pl0.copy() if tag else None
    orc, ocuts, orows = oracle.plan_tiers(counts, p, tiers, cap=cap, placement=o_pl)
    d_counts = torch.from_numpy(counts.view(np.int32)).to(G.DEV)
    d_rows = torch.full((max(cap, 1),), -1, dtype=torch.int64, device=G.DEV)
    d_cuts = torch.full((fs.FS_TIER_CUTS,), -1, dtype=torch.int64, device=G.DEV)
    d_pl = G.placement_dev(pl0) if tag else None
    rc = fs.fs_plan_tiers(d_counts, R, p, tiers, d_rows, cap, d_cuts, d_pl, raise_on_error=False)
    torch.cuda.synchronize()
    assert rc == orc
    if rc != 0:
        return rc, None
    cuts = d_cuts.cpu().numpy()
    assert cuts.tolist() == ocuts.tolist(), (cuts.tolist(), ocuts.tolist())
    k = min(cap, int(cuts[fs.FS_CUT_N_DP] + cuts[fs.FS_CUT_N_FLEX]))
    assert np.array_equal(d_rows.cpu().numpy()[:k], orows)
    assert torch.all(d_rows[k:] == -1)
    if tag:
        assert np.array_equal(d_pl.cpu().numpy().view(np.uint32), o_pl)
    return rc, cuts


@pytest.mark.parametrize("block", range(10))
def test_random_small(G, block):
    """Thirty random parameter sets per block: list lengths around the multiples of 64 and 4096, all-equal and
    mostly-zero counts, every tier count, capacities and with or without tags."""
    for seed in range(30 * block, 30 * block + 30):
        rng = np.random.default_rng(10_000 + seed)
        R = int(rng.choice([1, 2, 63, 64, 65, 4095, 4096, 4097, int(rng.integers(1, 60000))]))
        S = int(rng.integers(1, 6000))
        scale = int(rng.integers(1, 60))
        counts = np.minimum(rng.pareto(rng.choice([0.5, 0.8, 1.2, 2.0]), R) * scale, 4 * S).astype(np.uint32)
        counts[rng.random(R) < rng.choice([0.0, 0.2, 0.9])] = 0
        if rng.random() < 0.2:
            counts[:] = int(rng.integers(0, 5))
        U = int(rng.choice([1, 2, 4, 8, 32, 64]))
        W = int(rng.choice([w for w in (1, 2, 4, 8, 64) if U % w == 0]))
        p = params(num_samples=S, B=int(rng.integers(1, 600)), U=U, W=W, dp_multiplier=int(rng.integers(1, 9)),
                   granule=int(rng.choice([1, 2, 3, 32, 100])), a2a_global=int(rng.integers(1, 40)),
                   a2a_intra=int(rng.integers(1, 120)), ar_global=int(rng.integers(1, 120)), ar_cross=int(rng.integers(1, 80)))
        for tiers in (2, 3):
            both(G, counts, p, tiers, cap=int(rng.choice([R, 0, max(1, R // 3)])), tag=bool(rng.random() < 0.7))


def test_hand_case_and_edges(G):
    import paper_2301_02959_amd as fs
    counts = np.array([0, 300, 150, 143, 20, 10, 10, 5, 0, 1], np.uint32)
    p = params(num_samples=100, B=4, U=4, W=2, a2a_global=1, a2a_intra=4, ar_global=3, ar_cross=2)
    rc, cuts = both(G, counts, p, 3)
    assert cuts.tolist() == [8, 2, 4, 7, 7, 2, 2, 639, 450, 163]
    rc, cuts = both(G, counts, p, 2, cap=2)
    assert cuts[fs.FS_CUT_N_DP] == 4
    both(G, counts, dict(p, granule=3), 3)
    both(G, np.array([3000, 50, 50, 50, 50, 50, 50, 50], np.uint32), p, 3)
    both(G, np.array([3000, 150, 4, 4, 4, 4], np.uint32), p, 3)
    # no candidates, one candidate, everything replicated, nothing replicated
    rc, cuts = both(G, np.zeros(5000, np.uint32), p, 3)
    assert cuts.tolist() == [0] * 10
    both(G, np.array([0, 0, 9, 0], np.uint32), p, 2)
    both(G, np.full(4096 * 3, 1000, np.uint32), p, 2)
    both(G, np.full(4096 * 3 + 1, 1, np.uint32), p, 3)
    # a row exactly on the memory breakpoint
    both(G, np.array([7, 7, 6], np.uint32), params(num_samples=7, B=5, U=1, W=1), 2)
    # Flex is free (one group spans all GPUs, 1x static memory): limited by its traffic breakpoint only
    both(G, np.array([900, 800, 30, 20, 10, 5, 1], np.uint32), params(num_samples=100, B=4, U=4, W=4, dp_multiplier=1), 3)


@pytest.mark.parametrize("tiers", [2, 3])
@pytest.mark.parametrize("B", [64, 1024, 4096])
def test_power_law_many_tiles(G, tiers, B):
    # the cut at B (and the Flex budget) falls in different tiles of the summed counts as B changes
    rng = np.random.default_rng(B)
    R = 1_500_000
    z = 1.0 / np.arange(1, R + 1) ** 1.15
    S = 1 << 18
    counts = rng.permutation(np.floor(z / z.sum() * 700 * S)).astype(np.uint32)
    p = params(num_samples=S, B=B, U=32, W=8, granule=32, a2a_global=1, a2a_intra=6, ar_global=3, ar_cross=2)
    rc, cuts = both(G, counts, p, tiers)
    assert 0 < cuts[1] <= cuts[2] <= cuts[0]


@pytest.mark.parametrize("model", ["rm1", "rm3"])
def test_paper_tier_table_distribution(G, model):
    """The piecewise-constant distribution built from the paper's tier table (rows and average length
    divided by 32, which keeps every row probability): the GPU cuts it where the oracle does, which is
    where the paper did (the oracle's own test checks that part)."""
    from fractions import Fraction as Fr
    from test_oracle_plan import golden
    g = golden()
    U, W, dp, Bp = g["train_gpus"], g["train_gpus_per_node"], g["dp_static_multiplier"], g["rm1_local_batch"]
    E = g[f"{model}_rows"] // 32
    k2, kd, kf = (g[f"{model}_2tier_dp"] // 32, g[f"{model}_3tier_dp"] // 32, g[f"{model}_3tier_flex"] // 32)
    c2, cd, cf = (Fr(str(g[f"{model}_2tier_dp_cov_pct"])) / 100, Fr(str(g[f"{model}_3tier_dp_cov_pct"])) / 100,
                  Fr(str(g[f"{model}_3tier_flex_cov_pct"])) / 100)
    L = k2 * (dp - Fr(1, U)) / (Bp * c2)
    S = 1 << 30
    levels = [(kd, cd), (k2 - kd, c2 - cd), (kd + kf - k2, cd + cf - c2), (E - kd - kf, 1 - cd - cf)]
    counts = np.concatenate([np.full(n, int(round(cov * L / n * S)), np.uint32) for n, cov in levels])
    p = params(num_samples=S, B=Bp, U=U, W=W, dp_multiplier=dp, granule=1,
               a2a_global=1, a2a_intra=1000, ar_global=3, ar_cross=1000)
    rc, cuts2 = both(G, counts, p, 2, cap=0, tag=False)
    rc, cuts3 = both(G, counts, p, 3, tag=True)
    assert abs(int(cuts2[5]) - k2) <= 2 and cuts3[5] == kd and abs(int(cuts3[6]) - kf) <= 0.015 * kf


def test_host_faults(G):
    import paper_2301_02959_amd as fs
    counts = np.ones(4, np.uint32)
    for bad in (dict(num_samples=0), dict(U=8, W=3), dict(granule=0), dict(dp_multiplier=0), dict(ar_cross=0),
                dict(a2a_global=1 << 20), dict(B=0)):
        assert both(G, counts, params(**bad), 2)[0] == 6
    assert both(G, counts, params(), 4)[0] == 6
    assert both(G, counts, params(), 2, cap=-1)[0] == 2
    d = torch.zeros(4, dtype=torch.int32, device=G.DEV)
    cuts = torch.zeros(10, dtype=torch.int64, device=G.DEV)
    rows = torch.zeros(4, dtype=torch.int64, device=G.DEV)
    assert fs.fs_plan_tiers(None, 4, params(), 2, rows, 4, cuts, raise_on_error=False) == 1
    assert fs.fs_plan_tiers(d, 4, params(), 2, None, 4, cuts, raise_on_error=False) == 1
    assert fs.fs_plan_tiers(d, 4, params(), 2, rows, 4, None, raise_on_error=False) == 1
    assert fs.fs_plan_tiers(d, 0, params(), 2, rows, 4, cuts, raise_on_error=False) == 2
    small = torch.zeros(256, dtype=torch.uint8, device=G.DEV)
    assert fs.fs_plan_tiers(d, 4, params(), 2, rows, 4, cuts, workspace=small[:64], raise_on_error=False) == 5
    torch.cuda.synchronize()


def test_c3_profile_of_one_batch(G):
    """Counts of one c3 batch (accumulated by fs_plan_replication), tiers planned for the paper's
    training shape at this batch size; the plan's tags then drive fs_route_bucketize."""
    import paper_2301_02959_amd as fs
    cfg = fs_inputs.CONFIGS["c3"]
    b = fs_inputs.make_batch(cfg, G.DEV, keep_perms=False)
    n, R = b["n"], cfg.R
    counts = torch.zeros(R, dtype=torch.int32, device=G.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    fs.fs_plan_replication(b["ids"], b["offsets"], cfg.T, cfg.B, b["row_base"], n, R, counts, fs.FS_PLAN_ACCUMULATE,
                           dev_status=st)
    p = params(num_samples=cfg.B, B=cfg.B, U=cfg.U, W=cfg.W, granule=32, a2a_global=1, a2a_intra=6, ar_global=3,
               ar_cross=2)
    c_h = counts.cpu().numpy().view(np.uint32)
    for tiers in (2, 3):
        orc, ocuts, orows = oracle.plan_tiers(c_h, p, tiers)
        rows = torch.full((R,), -1, dtype=torch.int64, device=G.DEV)
        cuts = torch.zeros(fs.FS_TIER_CUTS, dtype=torch.int64, device=G.DEV)
        pl = torch.full((R,), entry(2, 5) - (1 << 32), dtype=torch.int32, device=G.DEV)     # the same 32 bits
        fs.fs_plan_tiers(counts, R, p, tiers, rows, R, cuts, pl, st)
        torch.cuda.synchronize()
        assert cuts.cpu().numpy().tolist() == ocuts.tolist()
        assert np.array_equal(rows[:len(orows)].cpu().numpy(), orows)
        n_dp, n_fx = int(cuts[fs.FS_CUT_N_DP]), int(cuts[fs.FS_CUT_N_FLEX])
        assert n_dp > 0 and int(cuts[fs.FS_CUT_SUM_ALL]) == n
        # the share of lookups the plan predicts for each tier is what routing then counts
        bo = torch.zeros(cfg.U + 1, dtype=torch.int64, device=G.DEV)
        r_o = torch.zeros(n, dtype=torch.int64, device=G.DEV)
        p_o = torch.zeros(n, dtype=torch.int32, device=G.DEV)
        tc = torch.zeros(3, dtype=torch.int64, device=G.DEV)
        fs.fs_route_bucketize(b["ids"], b["offsets"], cfg.T, cfg.B, b["row_base"], pl, n, cfg.U, cfg.W, cfg.self_bucket,
                              bo, r_o, p_o, tc, st)
        torch.cuda.synchronize()
        assert int(st.item()) == 0
        assert tc.tolist() == [int(cuts[fs.FS_CUT_SUM_DP]), int(cuts[fs.FS_CUT_SUM_FLEX]),
                               n - int(cuts[fs.FS_CUT_SUM_DP]) - int(cuts[fs.FS_CUT_SUM_FLEX])]


def test_breakpoints_at_every_position(G):
    """Points A and C on every index of the sorted candidates in turn (all of them for short lists, both ends and a
    stride for long ones): the 64-way searches must land exactly there, whatever the list length is modulo 64."""
    p = params(num_samples=100, B=4, U=4, W=2, dp_multiplier=6, granule=1,
               a2a_global=30, a2a_intra=40, ar_global=1, ar_cross=20)
    # smallest count at or above the breakpoint: A ceil(23 * 100 / 16) = 144, C ceil(30 * 100 / 8) = 375
    rng = np.random.default_rng(5)
    for K in (1, 2, 63, 64, 65, 66, 127, 128, 129, 381, 4095, 4096, 4097):
        where = range(K + 1) if K <= 129 else sorted(set(range(0, 70)) | set(range(K - 70, K + 1)) | set(range(0, K + 1, 97)))
        perm = rng.permutation(K)
        for F in where:
            for low, high in ((100, 200), (200, 400)):            # A at F (C nowhere); C at F (A everywhere)
                counts = np.full(K, low, np.uint32)
                counts[perm[:F]] = high
                rc, cuts = both(G, counts, p, 2, cap=0, tag=False)
                assert rc == 0
                if low == 100:
                    assert cuts[1] == F and cuts[3] == 0
                else:
                    assert cuts[1] == K and cuts[3] == F
