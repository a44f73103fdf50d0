"""Pins for the oracle's tier planner (Sections 4.2, 4.3, 4.5).

The planner walks rows in descending frequency order and cuts the walk at the breakpoints of the
per-row cost model (the cost tables of Section 3.2 with E = 1 and L = p).  It is pinned by
  * a brute force that never forms a marginal term: it evaluates the WHOLE memory and traffic of
    every prefix from the table formulas in exact fractions and reads the points off the curves
    (A = last minimum of memory, B = last prefix not above the all-row-wise memory, C = last
    minimum of traffic), and grows the Flex tier row by row against the same totals;
  * the row counts and coverage percentages the paper prints for its four models
    (tests/golden/paper_tables.txt): a piecewise-constant distribution built from those columns
    must be cut where the paper cut it;
  * closed forms (uniform distributions, rows exactly on a breakpoint, the 1/(6B) traffic
    breakpoint at all-reduce = 3 x all-to-all bandwidth) and invariants.
"""
from fractions import Fraction as Fr

import numpy as np
import pytest

import oracle
from helpers import entry
from test_oracle_plan import golden

C = oracle


def params(**kw):
    p = dict(num_samples=1000, B=16, U=8, W=4, dp_multiplier=6, granule=1,
             a2a_global=10, a2a_intra=40, ar_global=30, ar_cross=20)
    p.update(kw)
    return p


def brute(counts, p, tiers):
    """Whole-table costs per prefix from the table formulas, in exact fractions."""
    S, B, U, W, dp, gran = p["num_samples"], p["B"], p["U"], p["W"], p["dp_multiplier"], p["granule"]
    order = [g for g in np.lexsort((np.arange(len(counts)), -counts.astype(np.int64))) if counts[g] > 0]
    prob = [Fr(int(counts[g]), S) for g in order]
    K = len(order)

    def memory(n_dp, n_flex):
        tot = Fr(0)
        for i, q in enumerate(prob):
            if i < n_dp:
                tot += dp + B * q                      # static 6 E D dtype, dynamic B L D dtype, E = 1, L = p
            elif i < n_dp + n_flex:
                tot += Fr(dp, W) + 2 * B * q
            else:
                tot += Fr(1, U) + 2 * B * q
        return tot

    def traffic_dp(k):                                 # first k rows replicated, the rest row-wise
        return sum((Fr(1, p["ar_global"]) if i < k else 2 * B * q / p["a2a_global"]) for i, q in enumerate(prob))

    def traffic_flex(k):                               # first k rows Flex, the rest row-wise
        return sum((2 * B * q / p["a2a_intra"] + Fr(1, W * p["ar_cross"]) if i < k else 2 * B * q / p["a2a_global"])
                   for i, q in enumerate(prob))

    mem = [memory(k, 0) for k in range(K + 1)]
    kA = max(k for k in range(K + 1) if mem[k] == min(mem))
    kB = max(k for k in range(K + 1) if mem[k] <= mem[0])
    tr = [traffic_dp(k) for k in range(K + 1)]
    kC = max(k for k in range(K + 1) if tr[k] == min(tr))
    tf = [traffic_flex(k) for k in range(K + 1)]
    kF = max(k for k in range(K + 1) if tf[k] == min(tf))
    if tiers == 2:
        n_dp, n_flex = kB // gran * gran, 0
    else:
        n_dp = kA // gran * gran
        j = 0
        while n_dp + j < K and n_dp + j < kF and memory(n_dp, j + 1) <= mem[0]:
            j += 1
        n_flex = j // gran * gran
    return dict(K=K, kA=kA, kB=kB, kC=kC, kF=kF, n_dp=n_dp, n_flex=n_flex, order=order)


def check_against_brute(counts, p, tiers):
    rc, cuts, rows = C.plan_tiers(counts, p, tiers)
    b = brute(counts, p, tiers)
    assert rc == 0
    got = [int(cuts[i]) for i in (C.CUT_CANDIDATES, C.CUT_A, C.CUT_B, C.CUT_C, C.CUT_FLEX, C.CUT_N_DP, C.CUT_N_FLEX)]
    assert got == [b["K"], b["kA"], b["kB"], b["kC"], b["kF"], b["n_dp"], b["n_flex"]], (got, b)
    assert rows.tolist() == b["order"][:b["n_dp"] + b["n_flex"]]
    c64 = counts.astype(np.int64)
    assert cuts[C.CUT_SUM_ALL] == c64.sum()
    assert cuts[C.CUT_SUM_DP] == c64[b["order"][:b["n_dp"]]].sum()
    assert cuts[C.CUT_SUM_FLEX] == c64[b["order"][b["n_dp"]:b["n_dp"] + b["n_flex"]]].sum()
    return b


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("tiers", [2, 3])
def test_against_whole_curve_brute_force(seed, tiers):
    rng = np.random.default_rng(seed)
    R = int(rng.integers(5, 60))
    S = int(rng.integers(50, 400))
    counts = np.minimum(rng.pareto(0.7, R) * rng.integers(1, 30), 4 * S).astype(np.uint32)
    counts[rng.random(R) < 0.15] = 0
    counts[rng.integers(0, R, 3)] = counts[rng.integers(0, R, 3)]      # ties
    U = int(rng.choice([1, 2, 4, 8]))
    W = int(rng.choice([w for w in (1, 2, 4, 8) if U % w == 0]))
    p = params(num_samples=S, B=int(rng.integers(1, 40)), U=U, W=W, dp_multiplier=int(rng.integers(1, 8)),
               granule=int(rng.choice([1, 1, 2, 3])), a2a_global=int(rng.integers(1, 30)),
               a2a_intra=int(rng.integers(1, 90)), ar_global=int(rng.integers(1, 90)), ar_cross=int(rng.integers(1, 60)))
    check_against_brute(counts, p, tiers)


def test_three_tier_hand_case():
    # B = 4, U = 4, W = 2, 6x static memory, 100 samples: the memory breakpoint is (6 - 1/4) / 4 = 1.4375
    counts = np.array([0, 300, 150, 143, 20, 10, 10, 5, 0, 1], np.uint32)
    p = params(num_samples=100, B=4, U=4, W=2, a2a_global=1, a2a_intra=4, ar_global=3, ar_cross=2)
    rc, cuts, rows = C.plan_tiers(counts, p, 3)
    # rows by frequency: 1 (p=3), 2 (1.5), 3 (1.43), 4 (.2), 5, 6 (.1), 7 (.05), 9 (.01)
    # DP memory terms 5.75 - 4p: -6.25, -0.25, +0.03, ... -> A = 2; cumulative: -6.25, -6.5, -6.47, -1.52, 3.83 -> B = 4
    assert (cuts[C.CUT_CANDIDATES], cuts[C.CUT_A], cuts[C.CUT_B]) == (8, 2, 4)
    # DP traffic 1/3 - 8p <= 0  <=>  p >= 1/24: rows 1,2,3,4,5,6,7 -> C = 7
    assert cuts[C.CUT_C] == 7
    # Flex traffic 8p/4 + 1/(2*2) - 8p <= 0  <=>  p >= 1/24 -> FLEX = 7
    assert cuts[C.CUT_FLEX] == 7
    # three tiers: 2 DP rows save 6.5; a Flex row costs 6/2 - 1/4 = 2.75 -> 2 Flex rows (5.5 <= 6.5 < 8.25)
    assert (cuts[C.CUT_N_DP], cuts[C.CUT_N_FLEX]) == (2, 2) and rows.tolist() == [1, 2, 3, 4]
    assert (cuts[C.CUT_SUM_ALL], cuts[C.CUT_SUM_DP], cuts[C.CUT_SUM_FLEX]) == (639, 450, 163)
    rc, cuts2, rows2 = C.plan_tiers(counts, p, 2)
    assert (cuts2[C.CUT_N_DP], cuts2[C.CUT_N_FLEX]) == (4, 0) and rows2.tolist() == [1, 2, 3, 4]
    # the Flex tier stops at its traffic breakpoint even when memory is left: rows 3.. are below it
    rc, cuts3, rows3 = C.plan_tiers(np.array([3000, 150, 4, 4, 4, 4], np.uint32), p, 3)
    assert (cuts3[C.CUT_A], cuts3[C.CUT_FLEX], cuts3[C.CUT_N_DP], cuts3[C.CUT_N_FLEX]) == (2, 2, 2, 0)


def test_tags_and_rounding():
    counts = np.array([0, 300, 150, 143, 20, 10, 10, 5, 0, 1], np.uint32)
    p = params(num_samples=100, B=4, U=4, W=2, a2a_global=1, a2a_intra=4, ar_global=3, ar_cross=2)
    pl = np.full(10, entry(2, 3), np.uint32)
    rc, cuts, rows = C.plan_tiers(counts, p, 3, placement=pl)
    assert pl.tolist() == [entry(2, 3), entry(0, 3), entry(0, 3), entry(1, 0), entry(1, 1)] + [entry(2, 3)] * 5
    # more Flex rows than GPUs in a group: owners wrap around the group width, not the GPU count
    pl = np.full(8, entry(2, 0), np.uint32)
    rc, cuts, rows = C.plan_tiers(np.array([3000, 50, 50, 50, 50, 50, 50, 50], np.uint32), p, 3, placement=pl)
    assert (cuts[C.CUT_N_DP], cuts[C.CUT_N_FLEX]) == (1, 7)
    assert pl.tolist() == [entry(0, 0)] + [entry(1, i % 2) for i in range(7)]
    # granule 3: A = 2 -> 0 DP rows, nothing saved, no Flex rows; two tiers: B = 4 -> 3 rows
    rc, cuts, rows = C.plan_tiers(counts, dict(p, granule=3), 3)
    assert (cuts[C.CUT_A], cuts[C.CUT_N_DP], cuts[C.CUT_N_FLEX]) == (2, 0, 0) and len(rows) == 0
    rc, cuts, rows = C.plan_tiers(counts, dict(p, granule=3), 2)
    assert (cuts[C.CUT_B], cuts[C.CUT_N_DP]) == (4, 3) and rows.tolist() == [1, 2, 3]
    # the row list is cut at cap, the counts are not
    rc, cuts, rows = C.plan_tiers(counts, p, 2, cap=2)
    assert cuts[C.CUT_N_DP] == 4 and rows.tolist() == [1, 2]


def test_closed_forms():
    p = params(num_samples=(1 << 20) + 1, B=4096, U=32, W=8, a2a_global=1, a2a_intra=8, ar_global=3, ar_cross=3)
    S = p["num_samples"]
    p_mem = Fr(6 * 32 - 1, 32 * 4096)                        # (6 - 1/U) / B
    hot, cold = int(p_mem * S) + 1, int(p_mem * S)           # just above / just below the breakpoint
    # every row above the breakpoint: all replicated, at a saving; every row below: nothing is
    rc, cuts, _ = C.plan_tiers(np.full(500, hot, np.uint32), p, 2)
    assert (cuts[C.CUT_A], cuts[C.CUT_B], cuts[C.CUT_N_DP]) == (500, 500, 500)
    rc, cuts, _ = C.plan_tiers(np.full(500, cold, np.uint32), p, 2)
    assert (cuts[C.CUT_A], cuts[C.CUT_B], cuts[C.CUT_N_DP]) == (0, 0, 0)
    # a row exactly on the breakpoint is memory neutral: it belongs to A and to B
    q = params(num_samples=7, B=5, U=1, W=1, dp_multiplier=6)       # (6 - 1) / 5 = 1 = 7 / 7
    rc, cuts, _ = C.plan_tiers(np.array([7, 7, 6], np.uint32), q, 2)
    assert (cuts[C.CUT_A], cuts[C.CUT_B]) == (2, 2)
    # traffic breakpoint with all-reduce three times as fast as all-to-all: p = 1 / (6 B)
    on = S // (6 * 4096)
    assert S % (6 * 4096) != 0                                # so `on` is just below and on + 1 just above
    rc, cuts, _ = C.plan_tiers(np.array([on + 1, on + 1, on, on], np.uint32), p, 2)
    assert cuts[C.CUT_C] == 2
    # memory-neutral two-tier plan by hand: k hot rows at probability ph pay for j rows at pl
    ph, pl_ = 4 * hot, cold // 8
    save = (ph * 32 * 4096 - 191 * S) * 10                    # times U * S
    per_cold = 191 * S - pl_ * 32 * 4096
    j = save // per_cold
    rc, cuts, _ = C.plan_tiers(np.array([ph] * 10 + [pl_] * (j + 50), np.uint32), p, 2)
    assert (cuts[C.CUT_A], cuts[C.CUT_B]) == (10, 10 + j)
    # no faster link inside the node: Flex never beats row-wise on traffic
    rc, cuts, _ = C.plan_tiers(np.full(50, hot, np.uint32), dict(p, a2a_intra=1), 3)
    assert cuts[C.CUT_FLEX] == 0 and cuts[C.CUT_N_FLEX] == 0


@pytest.mark.parametrize("model", ["rm1", "rm2", "rm3", "rm4"])
def test_paper_tier_sizes(model):
    """A piecewise-constant distribution with the row counts and coverage columns of the paper's tier
    table must be cut where the paper cut it.  Rows and average length are both divided by 32, which
    leaves every per-row probability as it is (and the paper's tier sizes are multiples of 32)."""
    g = golden()
    U, W, dp, B = g["train_gpus"], g["train_gpus_per_node"], g["dp_static_multiplier"], g["rm1_local_batch"]
    scale = 32
    E = g[f"{model}_rows"] // scale
    k2, kd, kf = (g[f"{model}_2tier_dp"] // scale, g[f"{model}_3tier_dp"] // scale, g[f"{model}_3tier_flex"] // scale)
    assert all(g[f"{model}_{t}"] % scale == 0 for t in ("2tier_dp", "3tier_dp", "3tier_flex"))
    c2, cd, cf = (Fr(str(g[f"{model}_2tier_dp_cov_pct"])) / 100, Fr(str(g[f"{model}_3tier_dp_cov_pct"])) / 100,
                  Fr(str(g[f"{model}_3tier_flex_cov_pct"])) / 100)
    # the average length that makes the printed two-tier plan memory neutral: k (6 - 1/U) = B * coverage * L
    L = k2 * (dp - Fr(1, U)) / (B * c2)
    nominal = Fr(g[f"{model}_avg_length"], scale)
    assert abs(L - nominal) < Fr(6, 100) * nominal             # the paper's "~1000" / "~500"
    S = 1 << 30
    levels = [(kd, cd), (k2 - kd, c2 - cd), (kd + kf - k2, cd + cf - c2), (E - kd - kf, 1 - cd - cf)]
    counts = np.concatenate([np.full(n, int(round(cov * L / n * S)), np.uint32) for n, cov in levels])
    assert np.all(np.diff(counts.astype(np.int64)) <= 0)
    p = params(num_samples=S, B=B, U=U, W=W, dp_multiplier=dp, granule=1,
               a2a_global=1, a2a_intra=1000, ar_global=3, ar_cross=1000)     # traffic never limits the Flex tier
    rc, cuts, _ = C.plan_tiers(counts, p, 2)
    assert rc == 0 and abs(int(cuts[C.CUT_N_DP]) - k2) <= 2                   # rounding of the counts only
    rc, cuts, _ = C.plan_tiers(counts, p, 3)
    assert cuts[C.CUT_N_DP] == kd                                            # the printed DP tier ends at the breakpoint
    assert abs(int(cuts[C.CUT_N_FLEX]) - kf) <= 0.015 * kf                   # within 1.5 % of the printed Flex tier
    if model != "rm2":
        assert abs(int(cuts[C.CUT_N_FLEX]) - kf) <= 0.003 * kf
    cov_dp = cuts[C.CUT_SUM_DP] / cuts[C.CUT_SUM_ALL]
    assert abs(cov_dp - float(cd)) < 1e-3


def test_invariants_on_a_power_law():
    rng = np.random.default_rng(1)
    R = 200000
    z = 1.0 / np.arange(1, R + 1) ** 1.1
    S = 1 << 16
    counts = rng.permutation(np.floor(z / z.sum() * 300 * S)).astype(np.uint32)
    p = params(num_samples=S, B=256, U=32, W=8, granule=32, a2a_global=1, a2a_intra=6, ar_global=3, ar_cross=2)
    rc, c2, r2 = C.plan_tiers(counts, p, 2)
    rc, c3, r3 = C.plan_tiers(counts, p, 3)
    assert 0 < c2[C.CUT_A] <= c2[C.CUT_B] <= c2[C.CUT_C] <= c2[C.CUT_CANDIDATES]
    assert c2[C.CUT_N_DP] % 32 == 0 and c3[C.CUT_N_DP] % 32 == 0 and c3[C.CUT_N_FLEX] % 32 == 0
    assert c3[C.CUT_N_DP] <= c2[C.CUT_N_DP] <= c3[C.CUT_N_DP] + c3[C.CUT_N_FLEX]      # the Flex tier buys more rows
    srt = np.sort(counts.astype(np.int64))[::-1]

    def memory_terms(n_dp, n_flex):                                   # times U * S, plain integers
        dp_rows = sum((191 * S - 32 * 256 * int(c)) for c in srt[:n_dp])
        return dp_rows + n_flex * (6 * 4 - 1) * S
    assert memory_terms(int(c2[C.CUT_N_DP]), 0) <= 0 < memory_terms(int(c2[C.CUT_B]) + 1, 0)
    assert memory_terms(int(c3[C.CUT_N_DP]), int(c3[C.CUT_N_FLEX])) <= 0
    assert memory_terms(int(c3[C.CUT_N_DP]), int(c3[C.CUT_N_FLEX]) + 32) > 0 or \
        c3[C.CUT_N_DP] + c3[C.CUT_N_FLEX] + 32 > c3[C.CUT_FLEX]
    assert np.array_equal(counts[r3].astype(np.int64), srt[:len(r3)])                 # rows come in frequency order


def test_host_faults():
    counts = np.ones(4, np.uint32)
    assert C.plan_tiers(counts, params(), 4)[0] == 6
    assert C.plan_tiers(counts, params(num_samples=0), 2)[0] == 6
    assert C.plan_tiers(counts, params(U=8, W=3), 2)[0] == 6
    assert C.plan_tiers(counts, params(granule=0), 2)[0] == 6
    assert C.plan_tiers(counts, params(dp_multiplier=0), 2)[0] == 6
    assert C.plan_tiers(counts, params(ar_cross=0), 2)[0] == 6
    assert C.plan_tiers(counts, params(a2a_global=1 << 20), 2)[0] == 6
    assert C.plan_tiers(counts, params(), 2, cap=-1)[0] == 2
    rc, cuts, rows = C.plan_tiers(np.zeros(4, np.uint32), params(), 3)
    assert rc == 0 and cuts.tolist() == [0] * 10 and len(rows) == 0
