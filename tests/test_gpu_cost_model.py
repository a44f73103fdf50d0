"""Parity of the library's fs_cost_model / fs_tier_traffic (host arithmetic in double precision)
with the oracle's exact fractions: every cell of both cost tables within 1e-12 relative."""
import numpy as np
import pytest

from oracle import cost_model as cm

pytestmark = pytest.mark.gpu


def test_cost_tables_cell_by_cell():
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(0)
    cases = [dict(E=30_000_000, D=256, dtype_bytes=4, L=1000, W=8, N=4, B=4096, a2a_global=10**9, a2a_intra=8 * 10**9,
                  ar_global=3 * 10**9, ar_cross=2 * 10**9, dp_multiplier=6),
             dict(E=1, D=256, dtype_bytes=2, L=0.00145, W=8, N=8, B=8192, a2a_global=5e10, a2a_intra=4e11,
                  ar_global=1.5e11, ar_cross=9e10, dp_multiplier=6)]
    for _ in range(20):
        cases.append(dict(E=int(rng.integers(1, 10**8)), D=int(rng.choice([64, 128, 256, 512])),
                          dtype_bytes=int(rng.choice([1, 2, 4])), L=float(rng.uniform(0, 3000)),
                          W=int(rng.choice([1, 2, 4, 8])), N=int(rng.integers(1, 17)), B=int(rng.integers(1, 10**5)),
                          a2a_global=float(rng.uniform(1e8, 1e12)), a2a_intra=float(rng.uniform(1e8, 1e12)),
                          ar_global=float(rng.uniform(1e8, 1e12)), ar_cross=float(rng.uniform(1e8, 1e12)),
                          dp_multiplier=int(rng.integers(1, 8))))
    for p in cases:
        for strat in (cm.RW, cm.CW, cm.DP, cm.FLEX):
            code, got = fs.fs_cost_model(p, strat)
            want = [float(x) for x in cm.cost_model(p, strat)]
            assert code == 0
            assert np.allclose(got, want, rtol=1e-12, atol=0.0), (p, strat, got, want)
    assert fs.fs_cost_model(cases[0], 4, raise_on_error=False)[0] == 6
    assert fs.fs_cost_model(dict(cases[0], W=0), 0, raise_on_error=False)[0] == 6
    assert fs.fs_cost_model(dict(cases[0], L=float("nan")), 0, raise_on_error=False)[0] == 6


def test_tier_traffic():
    import paper_2301_02959_amd as fs
    for tc, D, s in (([14095415, 886213, 770096], 256, 2), ([0, 0, 5], 64, 4), ([7, 0, 0], 8, 1), ([0, 0, 0], 8, 2)):
        code, got = fs.fs_tier_traffic(tc, D, s)
        want = [float(x) for x in cm.tier_traffic(tc, D, s)]
        assert code == 0 and np.allclose(got, want, rtol=1e-12, atol=0.0)
    assert fs.fs_tier_traffic([1, -1, 0], 8, 2, raise_on_error=False)[0] == 2
    assert fs.fs_tier_traffic([1, 1, 0], 0, 2, raise_on_error=False)[0] == 2
